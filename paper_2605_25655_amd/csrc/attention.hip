// Decode attention on gfx950: one new token per request against that request's own key/value cache
// (Eq. 6, softmax(Q K^T / sqrt(d)) V per head; Sec. III-D.1: attention runs per request because every
// request has its own cache).  HBM-bound: K and V are read once.
//
// What is kept from the paper's MT Attention (Sec. III-C.2): Q and O stay on chip for the whole pass
// (registers here) while K and V are streamed by; the scores and weights of a block never leave the
// chip (stages 1-3 run back to back on a block of positions, with a running maximum and sum so that
// one pass suffices).  What is not: its row-block/outer-product tiling for scratchpads.
//
// Layout: q[B,Hq,D], k/v[B,Hkv,S_max,D] (one head's positions contiguous), out[B,Hq,D], all fp16;
// seq_lens[B] int32 on the device.  Query head h reads cache head h / (Hq/Hkv).
//
// Work split: a workgroup (4 waves) takes one chunk of positions of one (request, cache head) and up
// to GT query heads of that cache head's group.  16 (D = 128) or 8 (D = 64) lanes cover one row with
// 16-byte loads, so a wave instruction reads 4 or 8 consecutive positions = 1 KiB of contiguous memory;
// U such loads of K and of V are in flight per wave, one iteration ahead of the arithmetic.  A lane
// forms its 8-element share of q.k with packed fp16 dot products accumulated in fp32, the shares meet
// by lane shuffles, the weights stay fp32, and V is accumulated in fp32.  Row groups, waves and chunks
// each keep their own (maximum, sum, output) triple; triples are merged in a fixed order (row groups
// by shuffle, waves through LDS, chunks by a second small kernel), so results are reproducible.
#include "thi_internal.h"

namespace thi {

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int AT_THREADS = 256;
constexpr int AT_WAVES = 4;

template <int GT> struct Unroll { static constexpr int U = (GT >= 4) ? 2 : 4; };

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D, int GT>
__global__ __launch_bounds__(AT_THREADS) void attn_decode(AttnArgs a)
{
    constexpr int LPR = D / 8;                 // lanes per row
    constexpr int RG = 64 / LPR;               // rows (positions) per wave instruction
    constexpr int U = Unroll<GT>::U;           // wave instructions of K (and of V) per iteration
    constexpr int WPOS = RG * U;               // positions per wave and iteration
    constexpr int GPOS = AT_WAVES * WPOS;      // positions per workgroup and iteration
    __shared__ float s_o[AT_WAVES][GT][D];
    __shared__ float s_m[AT_WAVES][GT], s_l[AT_WAVES][GT];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int split = blockIdx.x, b = blockIdx.z;
    const int passes = (a.group + GT - 1) / GT;
    const int g = blockIdx.y / passes, pass = blockIdx.y % passes;
    const int L = a.seq_lens[b];
    const int c0 = split * a.chunk;
    const int c1 = (c0 + a.chunk < L) ? c0 + a.chunk : L;
    const int h0 = g * a.group + pass * GT;    // first query head of this workgroup
    const int heads = (a.group - pass * GT < GT) ? a.group - pass * GT : GT;
    if (c0 >= c1) {                            // nothing of this request in this chunk (uniform: no barrier yet)
        if (L == 0 && split == 0)              // an empty request: its output is zero
            for (int idx = tid; idx < heads * D; idx += AT_THREADS)
                a.out[((size_t)b * a.Hq + h0 + idx / D) * D + idx % D] = 0;
        return;
    }
    const int r = lane / LPR, piece = lane % LPR;

    // the query heads' 8-element shares, as fp16 pairs (zero for the heads past the group's end)
    half2_t qv[GT][4];
#pragma unroll
    for (int j = 0; j < GT; ++j) {
        uintx4 raw = {0u, 0u, 0u, 0u};
        if (j < heads) raw = *reinterpret_cast<const uintx4*>(a.q + ((size_t)(b * a.Hq + h0 + j)) * D + piece * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const unsigned w = raw[e];
            qv[j][e] = __builtin_bit_cast(half2_t, w);
        }
    }
    const uint16_t* kbase = a.k + ((size_t)(b * a.Hkv + g) * a.S_max) * D + piece * 8;
    const uint16_t* vbase = a.v + ((size_t)(b * a.Hkv + g) * a.S_max) * D + piece * 8;

    float m[GT], l[GT], o[GT][8];
#pragma unroll
    for (int j = 0; j < GT; ++j) {
        m[j] = -__builtin_inff();
        l[j] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[j][e] = 0.f;
    }

    // Loads are unconditional: a position past the chunk's end is redirected to the chunk's last row
    // (valid, cached) and its weight is forced to zero.
    auto issue = [&](int it, uintx4 (&kr)[U], uintx4 (&vr)[U]) {
        const int base = c0 + (it * AT_WAVES + wv) * WPOS;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int pos = base + u * RG + r;
            pos = pos < c1 ? pos : c1 - 1;
            kr[u] = ld_stream(kbase + (size_t)pos * D);
            vr[u] = ld_stream(vbase + (size_t)pos * D);
        }
    };

    const int n_it = (c1 - c0 + GPOS - 1) / GPOS;
    uintx4 kn[U], vn[U];
    issue(0, kn, vn);
    for (int it = 0; it < n_it; ++it) {
        uintx4 kc[U], vc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { kc[u] = kn[u]; vc[u] = vn[u]; }
        issue(it + 1, kn, vn);        // past the last iteration every lane is redirected to one cached row
        const int base = c0 + (it * AT_WAVES + wv) * WPOS;

        // stage 1: scores t[j][u] = scale2 * q_j . k_pos  (scale2 = scale * log2 e: weights via exp2)
        float t[GT][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            half2_t kp[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned w = kc[u][e];
                kp[e] = __builtin_bit_cast(half2_t, w);
            }
            const bool live = base + u * RG + r < c1;
#pragma unroll
            for (int j = 0; j < GT; ++j) {
                float acc = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_fdot2(kp[e], qv[j][e], acc, false);
#pragma unroll
                for (int sh = 1; sh < LPR; sh <<= 1) acc += __shfl_xor(acc, sh);
                t[j][u] = live ? acc * a.scale2 : -__builtin_inff();
            }
        }
        // stage 2: running maximum and sum, weights of this block
        float p[GT][U], corr[GT];
#pragma unroll
        for (int j = 0; j < GT; ++j) {
            float mb = t[j][0];
#pragma unroll
            for (int u = 1; u < U; ++u) mb = __builtin_fmaxf(mb, t[j][u]);
            const float mn = __builtin_fmaxf(m[j], mb);
            const float ms = (mn == -__builtin_inff()) ? 0.f : mn;     // nothing live yet: keep everything at zero
            corr[j] = exp2_fast(m[j] - ms);
            float sum = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) { p[j][u] = exp2_fast(t[j][u] - ms); sum += p[j][u]; }
            l[j] = l[j] * corr[j] + sum;
            m[j] = mn;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[j][e] *= corr[j];
        }
        // stage 3: weights times V (a dead position's V is zeroed so that 0 * garbage cannot leak)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool live = base + u * RG + r < c1;
            float vf[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned w = live ? vc[u][e] : 0u;
                const half2_t hv = __builtin_bit_cast(half2_t, w);
                vf[2 * e] = (float)hv[0];
                vf[2 * e + 1] = (float)hv[1];
            }
#pragma unroll
            for (int j = 0; j < GT; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) o[j][e] = __builtin_fmaf(p[j][u], vf[e], o[j][e]);
        }
    }

    // merge the row groups of the wave (fixed order: butterfly over the lane index)
#pragma unroll
    for (int sh = LPR; sh < 64; sh <<= 1) {
#pragma unroll
        for (int j = 0; j < GT; ++j) {
            const float m2 = __shfl_xor(m[j], sh), l2 = __shfl_xor(l[j], sh);
            const float mn = __builtin_fmaxf(m[j], m2);
            const float ms = (mn == -__builtin_inff()) ? 0.f : mn;
            const float ca = exp2_fast(m[j] - ms), cb = exp2_fast(m2 - ms);
            l[j] = l[j] * ca + l2 * cb;
            m[j] = mn;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float o2 = __shfl_xor(o[j][e], sh);
                o[j][e] = o[j][e] * ca + o2 * cb;
            }
        }
    }
    // the waves meet in LDS
    if (r == 0) {
#pragma unroll
        for (int j = 0; j < GT; ++j) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s_o[wv][j][piece * 8 + e] = o[j][e];
            if (piece == 0) { s_m[wv][j] = m[j]; s_l[wv][j] = l[j]; }
        }
    }
    __syncthreads();
    for (int idx = tid; idx < heads * D; idx += AT_THREADS) {
        const int j = idx / D, d = idx % D;
        float mn = s_m[0][j];
#pragma unroll
        for (int w = 1; w < AT_WAVES; ++w) mn = __builtin_fmaxf(mn, s_m[w][j]);
        const float ms = (mn == -__builtin_inff()) ? 0.f : mn;
        float lf = 0.f, of = 0.f;
#pragma unroll
        for (int w = 0; w < AT_WAVES; ++w) {        // fixed order: waves 0..3
            const float cw = exp2_fast(s_m[w][j] - ms);
            lf += s_l[w][j] * cw;
            of += s_o[w][j][d] * cw;
        }
        const size_t bh = (size_t)b * a.Hq + h0 + j;
        if (a.nsplit == 1) {
            a.out[bh * D + d] = to_half_bits(of / lf);       // lf > 0: the chunk holds at least one live position
        } else {
            float* po = a.part + (bh * a.nsplit + split) * (D + 2);
            po[d] = of;
            if (d == 0) { po[D] = mn; po[D + 1] = lf; }
        }
    }
}

// Grouped-query variant (D = 128, 4 or 8 query heads per cache head and pass): with several heads per
// key row the lane-shuffle dot products of attn_decode make the vector ALU the bottleneck, so the scores
// of 16 positions x up to 16 heads come from four v_mfma_f32_16x16x32_f16 (keys loaded straight into the
// A-operand layout: lane = (position, 8-element k group); queries resident as the B operand).  A lane
// then owns the scores of one head at four positions; the running maximum is shared by the four lanes of
// a head after every block, so all accumulators of a wave refer to the same maximum and merge by plain
// addition.  The weights reach the lanes that accumulate V (lane = (row group, 16-byte piece), positions
// 4 * row group + u) as fp16 pairs through one lane permutation per head and pair of positions; V stays on
// the vector ALU (packed fp16 dot products into fp32), two positions per instruction.
template <int GT>
__global__ __launch_bounds__(AT_THREADS) void attn_decode_gqa(AttnArgs a)
{
    constexpr int D = 128;
    constexpr int WPOS = 16, GPOS = AT_WAVES * WPOS;
    __shared__ float s_o[AT_WAVES][GT][D];
    __shared__ float s_m[AT_WAVES][GT], s_l[AT_WAVES][GT];
    __shared__ uintx4 s_q[4][64];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int split = blockIdx.x, b = blockIdx.z;
    const int passes = (a.group + GT - 1) / GT;
    const int g = blockIdx.y / passes, pass = blockIdx.y % passes;
    const int L = a.seq_lens[b];
    const int c0 = split * a.chunk;
    const int c1 = (c0 + a.chunk < L) ? c0 + a.chunk : L;
    const int h0 = g * a.group + pass * GT;
    const int heads = (a.group - pass * GT < GT) ? a.group - pass * GT : GT;
    if (c0 >= c1) {
        if (L == 0 && split == 0)
            for (int idx = tid; idx < heads * D; idx += AT_THREADS)
                a.out[((size_t)b * a.Hq + h0 + idx / D) * D + idx % D] = 0;
        return;
    }
    const int lo = lane & 15, hi = lane >> 4;      // scores: (head column, position quad); V: (piece, row group)

    // B operand (head lo, k group hi, per 32-wide k step), kept in LDS: every wave reads the same
    if (wv == 0) {
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            uintx4 raw = {0u, 0u, 0u, 0u};
            if (lo < heads) raw = *reinterpret_cast<const uintx4*>(a.q + ((size_t)(b * a.Hq + h0 + lo)) * D + s4 * 32 + hi * 8);
            s_q[s4][lane] = raw;
        }
    }
    __syncthreads();
    const uint16_t* kbase = a.k + ((size_t)(b * a.Hkv + g) * a.S_max) * D;
    const uint16_t* vbase = a.v + ((size_t)(b * a.Hkv + g) * a.S_max) * D + lo * 8;

    float m = -__builtin_inff(), l = 0.f;           // of head lo (l: this lane's four positions only)
    float o[GT][8];
#pragma unroll
    for (int j = 0; j < GT; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[j][e] = 0.f;

    auto issue_k = [&](int it, uintx4 (&kr)[4]) {
        const int base = c0 + (it * AT_WAVES + wv) * WPOS;
        int kp = base + lo;                          // A operand: row lo of the block
        kp = kp < c1 ? kp : c1 - 1;
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) kr[s4] = ld_stream(kbase + (size_t)kp * D + s4 * 32 + hi * 8);
    };
    auto issue_v = [&](int it, uintx4 (&vr)[4]) {
        const int base = c0 + (it * AT_WAVES + wv) * WPOS;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int vp = base + 4 * hi + u;
            vp = vp < c1 ? vp : c1 - 1;
            vr[u] = ld_stream(vbase + (size_t)vp * D);
        }
    };

    const int n_it = (c1 - c0 + GPOS - 1) / GPOS;
    // Register budget (three waves per SIMD need <= 168): the keys of the next block are requested only
    // after this block's score MFMAs have consumed the current ones (same registers), the values are
    // one block ahead, and the queries are re-read from LDS as the B operand.
    uintx4 kreg[4], vn[4];
    issue_k(0, kreg);
    issue_v(0, vn);
    for (int it = 0; it < n_it; ++it) {
        uintx4 vc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) vc[u] = vn[u];
        issue_v(it + 1, vn);
        const int base = c0 + (it * AT_WAVES + wv) * WPOS;

        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, kreg[s4]),
                                                         __builtin_bit_cast(half8, s_q[s4][lane]), acc, 0, 0, 0);
        issue_k(it + 1, kreg);
        float t[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = (base + 4 * hi + i < c1) ? acc[i] * a.scale2 : -__builtin_inff();
        float mb = __builtin_fmaxf(__builtin_fmaxf(t[0], t[1]), __builtin_fmaxf(t[2], t[3]));
        mb = __builtin_fmaxf(mb, __shfl_xor(mb, 16));
        mb = __builtin_fmaxf(mb, __shfl_xor(mb, 32));
        const float mn = __builtin_fmaxf(m, mb);
        const float ms = (mn == -__builtin_inff()) ? 0.f : mn;
        const float corr = exp2_fast(m - ms);
        float p[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) p[i] = exp2_fast(t[i] - ms);
        l = l * corr + ((p[0] + p[1]) + (p[2] + p[3]));
        m = mn;
        // the accumulators are rescaled only when some head's maximum moved (rare after the first blocks)
        if (__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0ull) {
#pragma unroll
            for (int j = 0; j < GT; ++j) {
                const float cj = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, corr), j));
#pragma unroll
                for (int e = 0; e < 8; ++e) o[j][e] *= cj;
            }
        }
        // weights times V, two positions per instruction: v_dot2_f32_f16 on (V[u][d], V[u+1][d]) and the
        // fp16 pair of their weights (weights are in [0,1]: 2^-11 relative rounding), fp32 accumulation
        half2_t ppair[2];
        ppair[0] = half2_t{(_Float16)p[0], (_Float16)p[1]};
        ppair[1] = half2_t{(_Float16)p[2], (_Float16)p[3]};
#pragma unroll
        for (int up = 0; up < 2; ++up) {
            const bool live0 = base + 4 * hi + 2 * up < c1, live1 = base + 4 * hi + 2 * up + 1 < c1;
            half2_t vpk[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned w0 = live0 ? vc[2 * up][e] : 0u, w1 = live1 ? vc[2 * up + 1][e] : 0u;
                vpk[2 * e] = __builtin_bit_cast(half2_t, __builtin_amdgcn_perm(w1, w0, 0x05040100u));
                vpk[2 * e + 1] = __builtin_bit_cast(half2_t, __builtin_amdgcn_perm(w1, w0, 0x07060302u));
            }
#pragma unroll
            for (int j = 0; j < GT; ++j) {
                // head j's weights of positions 4*hi + 2*up and + 1 (held by lane j of this row group)
                const int bits = __shfl(__builtin_bit_cast(int, ppair[up]), j + 16 * hi);
                const half2_t pj = __builtin_bit_cast(half2_t, bits);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[j][e] = __builtin_amdgcn_fdot2(vpk[e], pj, o[j][e], false);
            }
        }
    }

    // the wave's four row groups: same maximum, so sums simply add
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
#pragma unroll
    for (int j = 0; j < GT; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            o[j][e] += __shfl_xor(o[j][e], 16);
            o[j][e] += __shfl_xor(o[j][e], 32);
        }
    if (hi == 0) {
#pragma unroll
        for (int j = 0; j < GT; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) s_o[wv][j][lo * 8 + e] = o[j][e];
        if (lo < GT) { s_m[wv][lo] = m; s_l[wv][lo] = l; }
    }
    __syncthreads();
    for (int idx = tid; idx < heads * D; idx += AT_THREADS) {
        const int j = idx / D, d = idx % D;
        float mn = s_m[0][j];
#pragma unroll
        for (int w = 1; w < AT_WAVES; ++w) mn = __builtin_fmaxf(mn, s_m[w][j]);
        const float ms = (mn == -__builtin_inff()) ? 0.f : mn;
        float lf = 0.f, of = 0.f;
#pragma unroll
        for (int w = 0; w < AT_WAVES; ++w) {        // fixed order: waves 0..3
            const float cw = exp2_fast(s_m[w][j] - ms);
            lf += s_l[w][j] * cw;
            of += s_o[w][j][d] * cw;
        }
        const size_t bh = (size_t)b * a.Hq + h0 + j;
        if (a.nsplit == 1) {
            a.out[bh * D + d] = to_half_bits(of / lf);
        } else {
            float* po = a.part + (bh * a.nsplit + split) * (D + 2);
            po[d] = of;
            if (d == 0) { po[D] = mn; po[D + 1] = lf; }
        }
    }
}

// Second pass when the positions were cut into chunks: one workgroup per (request, query head) merges
// the chunks' triples in chunk order and normalises.
template <int D>
__global__ __launch_bounds__(D) void attn_combine(AttnArgs a)
{
    const int bh = blockIdx.x, d = threadIdx.x;
    const int b = bh / a.Hq;
    const int L = a.seq_lens[b];
    const int live = (L + a.chunk - 1) / a.chunk;       // chunks that hold positions of this request
    float m = -__builtin_inff(), l = 0.f, o = 0.f;
    for (int s = 0; s < live; ++s) {
        const float* po = a.part + ((size_t)bh * a.nsplit + s) * (D + 2);
        const float m2 = po[D], l2 = po[D + 1], o2 = po[d];
        const float mn = __builtin_fmaxf(m, m2);
        const float ca = exp2_fast(m - mn), cb = exp2_fast(m2 - mn);      // m2 is finite: the chunk was live
        l = l * ca + l2 * cb;
        o = o * ca + o2 * cb;
        m = mn;
    }
    if (live > 0) a.out[(size_t)bh * D + d] = to_half_bits(o / l);      // (an empty request was zeroed by the first pass)
}

template <int D, int GT>
void launch_decode(const AttnArgs& a, dim3 grid, hipStream_t stream)
{
    hipLaunchKernelGGL((attn_decode<D, GT>), grid, dim3(AT_THREADS), 0, stream, a);
}

template <int D>
hipError_t launch_d(const AttnArgs& a, int gt, hipStream_t stream)
{
    const int passes = (a.group + gt - 1) / gt;
    dim3 grid((unsigned)a.nsplit, (unsigned)(a.Hkv * passes), (unsigned)a.B);
    switch (gt) {
    case 1: launch_decode<D, 1>(a, grid, stream); break;
    case 2: launch_decode<D, 2>(a, grid, stream); break;
    case 4:
        if (D == 128) hipLaunchKernelGGL((attn_decode_gqa<4>), grid, dim3(AT_THREADS), 0, stream, a);
        else launch_decode<D, 4>(a, grid, stream);
        break;
    default:
        if (D == 128) hipLaunchKernelGGL((attn_decode_gqa<8>), grid, dim3(AT_THREADS), 0, stream, a);
        else launch_decode<D, 8>(a, grid, stream);
        break;
    }
    if (a.nsplit > 1)
        hipLaunchKernelGGL((attn_combine<D>), dim3((unsigned)(a.B * a.Hq)), dim3(D), 0, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attention(const AttnArgs& a, hipStream_t stream)
{
    const int gt = attention_heads_per_workgroup(a.group);
    if (a.D == 128) return launch_d<128>(a, gt, stream);
    if (a.D == 64) return launch_d<64>(a, gt, stream);
    return hipErrorInvalidValue;
}

}  // namespace thi
