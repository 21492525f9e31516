// LDS-tiled fp16 MFMA GEMM for prefill (large M) on gfx950.
//
// Function: the paper's large-M linear operator (Sec. III-B.2) -- out = x W^T
// with fp16 operands and fp32 accumulation (Sec. III-B.4) -- plus the fused
// low-density operators behind it (Sec. III-C.1): SiLU(gate)*up, the rotary
// embedding, the residual.  RMSNorm in front runs as a small pass of its own
// (rmsnorm_rows below) so that both operand tiles can go from memory straight
// into LDS; fused into the staging of the activation tile it cost 25 % and
// three times the HBM reads.
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
// Scheduling: a fixed number of workgroups (one or two per CU).  Tiles that fill whole rounds of the
// grid are computed and finished in one piece; the ragged remainder (everything, when there are fewer
// tiles than workgroups) may be cut along K so that no CU idles -- into equal k ranges per tile, the
// same for every tile, when there are several token tiles (workgroups on neighbouring tiles then walk
// the same k range together and keep sharing operand panels through the L2), into equal contiguous
// stream-K shares when there is one token tile (every weight panel is read once anyway).  Tiles that
// were cut leave fp32 partial tiles in the workspace; a second, chip-wide kernel adds them in workgroup
// order (bitwise reproducible) and applies the epilogue.
//
// Workgroups are numbered so that the eight XCDs (one L2 each; hardware deals
// consecutive workgroup ids round-robin to them) each walk a contiguous range
// of tiles, token-tile fastest, so the weight panel an XCD streams is shared by
// the workgroups running on it at that moment.
#include "thi_internal.h"

#include <mutex>
#include <type_traits>

namespace thi {

namespace {

// A staged tile row holds GK halfs = GK/8 16-byte pieces.  Piece p of tile row `row` lives at 16-byte
// unit row*P + (p ^ f(row)), with f chosen so that 16 consecutive rows reading the same logical piece
// (an MFMA operand read) and the linear staging writes both spread over all LDS banks:
//   P = 8 (128-byte rows): f is a bijection on every aligned group of 8 rows and on the even and the odd
//                          rows of every aligned group of 16;
//   P = 4 (64-byte rows):  f is a bijection on {r, r+4, r+8, r+12} and on {r, r+2, r+4, r+6}.
template <int P>
__device__ __forceinline__ int swz_f(int row)
{
    if (P == 16) return row & 15;     // 256-byte rows: 16 consecutive rows, 16 different pieces
    if (P == 8) return ((row >> 1) & 7) ^ ((row & 1) << 2);
    return (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1);
}
template <int P>
__device__ __forceinline__ int swz(int row, int piece) { return row * P + (piece ^ swz_f<P>(row)); }

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

// The same load with the address split into a wave-uniform base (scalar registers) and a 32-bit
// per-lane byte offset: no vector ALU work per load.  Written in assembly because the builtin always
// takes the 64-bit per-lane form.  The kernels that use it use M0 for nothing else and wait for these
// loads explicitly (s_waitcnt vmcnt) before the barrier that publishes the stage.
__device__ __forceinline__ void dma16_sbase(const void* base_uniform, unsigned lane_byte_offset, uintx4* lds_base)
{
    const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)lds_base;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_byte_offset), "s"(base_uniform), "s"(lds_addr)
                 : "memory");
}

// The k-steps of the shared tiles (tile t = units [t * ktiles, (t + 1) * ktiles)) dealt to G workers.
//   parts == 0: contiguous equal shares whatever the tile boundaries (the first `rem` workers take q + 1
//               units, the others q); a share may span the end of one tile and the start of the next.
//   parts >= 1: every shared tile is cut into `parts` equal k ranges, worker w takes range w % parts of
//               tile w / parts (workers past sk_tiles * parts take none).  Workers on neighbouring tiles
//               then walk the same k range at the same time, so the operand panels they have in common
//               are still fetched once per L2 instead of once per workgroup.
struct Deal {
    int q, rem, parts, ktiles, shared;
    __device__ __forceinline__ Deal(int sk_tiles, int ktiles_, int G, int parts_)
        : q(sk_tiles * ktiles_ / G), rem(sk_tiles * ktiles_ % G), parts(parts_), ktiles(ktiles_), shared(sk_tiles) {}
    __device__ __forceinline__ int begin(int w) const {
        if (parts == 0) return w * q + (w < rem ? w : rem);
        if (w >= shared * parts) return shared * ktiles;
        return (w / parts) * ktiles + (w % parts) * ktiles / parts;
    }
    __device__ __forceinline__ int end(int w) const {
        if (parts == 0) return begin(w + 1);
        if (w >= shared * parts) return shared * ktiles;
        return (w / parts) * ktiles + (w % parts + 1) * ktiles / parts;
    }
    // first and last worker with a share of tile t
    __device__ __forceinline__ int first(int t) const { return parts == 0 ? owner(t * ktiles) : t * parts; }
    __device__ __forceinline__ int last(int t) const { return parts == 0 ? owner(t * ktiles + ktiles - 1) : t * parts + parts - 1; }
    __device__ __forceinline__ int owner(int u) const {
        const int edge = rem * (q + 1);
        return u < edge ? u / (q + 1) : rem + (u - edge) / q;
    }
};

// Epilogue for one 32x32 accumulator fragment: lane (lr = token within the fragment, lg = which
// half of the rows) holds, per register quad aa, four consecutive n of one token.
template <int BN, int BM, int WN, int WM, int EPI>
__device__ __forceinline__ void store_fragment(const GemmArgs& a, int tile_n, int tile_m, int wn, int wm, int tn,
                                               int tm, int lr, int lg, const floatx16& f,
                                               int aa_begin = 0, int aa_end = 4)
{
    constexpr int JPT = is_swiglu(EPI) ? BN / 2 : BN;
    const int m = tile_m * BM + wm * (BM / WM) + tm * 32 + lr;
    if (m >= a.M) return;
    if (is_swiglu(EPI)) {
#pragma unroll
        for (int aa = 0; aa < 4; aa += 2) {
            if (aa < aa_begin || aa >= aa_end) continue;
            const int v = wn * (BN / WN) + tn * 32 + 8 * aa;
            const int j = tile_n * JPT + (v >> 4) * 8 + 4 * lg;
            half4 hv;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float g = f[4 * aa + c], uu = f[4 * (aa + 1) + c];
                hv[c] = (_Float16)(g / (1.0f + __expf(-g)) * uu);
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
            if (aa < aa_begin || aa >= aa_end) continue;
            const int n = tile_n * BN + wn * (BN / WN) + tn * 32 + 8 * aa + 4 * lg;
            float v[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = f[4 * aa + c];
            if (has_rope(EPI)) {                         // the quad holds two complete pairs of one token
                if (EPI == EPI_ROPE) {                   // cos / sin from the table the RMSNorm pass left
                    rope_pair_table(a.rope, m, n, v[0], v[1]);
                    rope_pair_table(a.rope, m, n + 2, v[2], v[3]);
                } else {
                    const int mp = a.rope.pos[m];
                    rope_pair(a.rope, mp, n, v[0], v[1]);
                    rope_pair(a.rope, mp, n + 2, v[2], v[3]);
                }
            }
            if (n + 3 < a.N && (a.ldo & 3) == 0) {
                half4 hv;
                if (a.residual) {
                    const half4 rv = *reinterpret_cast<const half4*>(a.residual + (size_t)m * a.ldo + n);
#pragma unroll
                    for (int c = 0; c < 4; ++c) v[c] += (float)rv[c];
                }
#pragma unroll
                for (int c = 0; c < 4; ++c) hv[c] = (_Float16)v[c];
                *reinterpret_cast<half4*>(a.out + (size_t)m * a.ldo + n) = hv;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (n + c < a.N) {
                        if (a.residual) v[c] += half_bits_to_float(a.residual[(size_t)m * a.ldo + n + c]);
                        a.out[(size_t)m * a.ldo + n + c] = to_half_bits(v[c]);
                    }
            }
        }
    }
}

// Second pass for tiles that were cut along K: one workgroup per (shared tile, accumulator fragment, half of the
// fragment's register quads) adds the partial fragments of the tile's contributors in workgroup order
// and applies the epilogue.  The thread <-> element mapping is the main kernel's, so the partials are
// read back as they were written.  (Halves, not quads: SwiGLU pairs quad 2i with quad 2i+1.)
template <int BN, int BM, int WN, int WM, int EPI>
__global__ __launch_bounds__(64 * WN * WM) void gemm_fixup(GemmArgs a, int tiles_m, int ktiles, int sk_tiles, int G, int parts)
{
    constexpr int THREADS = 64 * WN * WM;
    constexpr int TN = BN / WN / 32, TM = BM / WM / 32;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid / 64;
    const int wn = wv % WN, wm = wv / WN, lr = lane & 31, lg = lane >> 5;
    const int half = blockIdx.x & 1, tf = blockIdx.x >> 1;
    const int t = tf / (TN * TM), frag = tf % (TN * TM);
    const int tn = frag / TM, tm = frag % TM;
    const Deal deal(sk_tiles, ktiles, G, parts);
    const int w_first = deal.first(t), w_last = deal.last(t);
    floatx4 g0 = {0.f, 0.f, 0.f, 0.f}, g1 = {0.f, 0.f, 0.f, 0.f};      // this half's two register quads
    // a contributor's partial of this tile: slot 0 if the tile is the first of its share, else slot 1
    auto part = [&](int wc) -> const floatx4* {
        const int cslot = (deal.begin(wc) / ktiles == t) ? 0 : 1;
        return reinterpret_cast<const floatx4*>(a.partials + ((size_t)wc * 2 + cslot) * (BN * BM)) +
               (frag * 4 + 2 * half) * THREADS + tid;
    };
    auto add = [&](const floatx4& v0, const floatx4& v1) { g0 += v0; g1 += v1; };
    int wc = w_first;
    for (; wc + 3 <= w_last; wc += 4) {      // four contributors' loads in flight, added in order
        const floatx4 *p0 = part(wc), *p1 = part(wc + 1), *p2 = part(wc + 2), *p3 = part(wc + 3);
        const floatx4 a0 = p0[0], a1 = p0[THREADS], b0 = p1[0], b1 = p1[THREADS];
        const floatx4 c0 = p2[0], c1 = p2[THREADS], d0 = p3[0], d1 = p3[THREADS];
        add(a0, a1); add(b0, b1); add(c0, c1); add(d0, d1);
    }
    for (; wc <= w_last; ++wc) {
        const floatx4* p = part(wc);
        const floatx4 v0 = p[0], v1 = p[THREADS];
        add(v0, v1);
    }
    floatx16 f;
#pragma unroll
    for (int e = 0; e < 16; ++e) f[e] = 0.f;
    if (half == 0) {
#pragma unroll
        for (int c = 0; c < 4; ++c) { f[c] = g0[c]; f[4 + c] = g1[c]; }
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) { f[8 + c] = g0[c]; f[12 + c] = g1[c]; }
    }
    store_fragment<BN, BM, WN, WM, EPI>(a, t / tiles_m, t % tiles_m, wn, wm, tn, tm, lr, lg, f, 2 * half, 2 * half + 2);
}

// BN x BM output tile, WN x WM waves; wave tile (BN/WN) x (BM/WM) built from 32x32 MFMA tiles.
// KTAIL: K is not a multiple of 64 (pieces past K are zero-filled; operands then go through VGPRs).
// FD: how many k-steps ahead of the MFMAs the operand fragments are read from LDS (1: two fragment buffers;
// 2: three, the 256x256 configuration).  The two waves of a SIMD do not share the matrix pipe evenly -- the
// older one is served first, finishes its k-tile early and waits at the barrier, and the other then runs
// alone, with MFMA blocks of 256 cycles per k-step instead of 512 to hide its LDS reads behind (cycle counters
// in the loop, 2048 x 8192 x 28672: the waves 0..3 waited ~1100 cycles per k-tile at the barrier, the waves 4..7
// ~170; the wait for the direct loads was 40..80 cycles).  One more k-step of distance gives the wave that runs
// alone more slack: 2757 -> 2625 cycles per k-tile (2048 would be the matrix pipe's own time), +2.2 % in
// throughput -- the clock gives back half of what the cycles gain.
template <int BN, int BM, int WN, int WM, int GK, int NS, int EPI, bool KTAIL, int FD = 1>
__global__ __launch_bounds__(64 * WN * WM) void gemm_streamk(GemmArgs a, int tiles_m, int ktiles, int sk_tiles, int parts)
{
    constexpr int NWAVES = WN * WM;
    constexpr int THREADS = 64 * NWAVES;
    constexpr int GPIECES = GK / 8;             // 16-byte pieces per tile row
    constexpr int KSTEPS = GK / 16;             // MFMA k-steps per staged tile (even)
    constexpr int ROWS_PER_DMA = 64 / GPIECES;  // tile rows covered by one wave-wide direct load
    constexpr int ROWS_PER_PASS = THREADS / GPIECES;
    constexpr int WPASS = BN / ROWS_PER_PASS;   // per-thread pieces of the weight tile
    constexpr int XPASS = BM / ROWS_PER_PASS;
    constexpr int TN = BN / WN / 32;            // MFMA tiles per wave along n
    constexpr int TM = BM / WM / 32;
    constexpr int JPT = is_swiglu(EPI) ? BN / 2 : BN;   // physical weight rows per tile
    constexpr bool W_DMA = !KTAIL;                           // weight tile: global -> LDS directly
    constexpr bool X_DMA = !KTAIL;                           // activation tile: the same
    constexpr int STAGE = (BN + BM) * GPIECES;   // 16-byte units per stage: weight tile, then activation tile
    // A direct weight load takes a wave-uniform base; with SwiGLU and 16 tile rows per load (GK = 32) one
    // load spans a gate block and an up block, so that variant keeps per-lane 64-bit addresses.
    constexpr bool W_SBASE = !(is_swiglu(EPI) && ROWS_PER_DMA != 8);
    static_assert(NS >= 2 && NS <= 8 && (KSTEPS % 2) == 0, "pipeline shape");
    static_assert(WPASS >= 1 && XPASS >= 1, "tile too small for the thread count");

    extern __shared__ uintx4 smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid / 64);     // wave index, known uniform to the compiler
    const int wn = wv % WN, wm = wv / WN;
    const int lr = lane & 31, lg = lane >> 5;
    const int K = a.K;

    // XCD-aware worker numbering: consecutive workers (neighbouring tiles) share an XCD
    const int G = gridDim.x;
    int worker;
    {
        const int bid = blockIdx.x, per = G / 8, rem = G % 8, xcd = bid % 8, local = bid / 8;
        worker = xcd * per + (xcd < rem ? xcd : rem) + local;
    }
    // The first sk_tiles tiles are cut along K and dealt as `Deal` says; the others are taken whole,
    // round-robin.  The shared tiles come first: their partial tiles are long written when the kernel ends.
    const Deal deal(sk_tiles, ktiles, G, parts);
    const int u_begin = deal.begin(worker), u_end = deal.end(worker);
    const int first_tile = u_begin / ktiles;
    int t_whole = sk_tiles + worker;

    // DMA staging role.  A wave instruction covers ROWS_PER_DMA tile rows = 64 consecutive LDS units;
    // lane L owns unit L of it: row (ROWS_PER_DMA*block + L/P), physical slot L%P, logical piece
    // slot ^ f(row).  VGPR staging role (operands that are zero-padded: ragged K): logical piece
    // tid%P of rows tid/P + ROWS_PER_PASS*i.
    const int slot = lane % GPIECES;
    const int vp = tid % GPIECES, vr0 = tid / GPIECES;
    const uintx4 zero4 = {0u, 0u, 0u, 0u};

    for (int u = u_begin;;) {
        int t, kb, ke;
        if (u < u_end) {
            t = u / ktiles;
            kb = u - t * ktiles;
            ke = (ktiles - kb < u_end - u) ? ktiles : kb + (u_end - u);
            u += ke - kb;
        } else if (t_whole < a.tiles) {
            t = t_whole;
            kb = 0;
            ke = ktiles;
            t_whole += G;
        } else {
            break;
        }
        const int tile_m = t % tiles_m, tile_n = t / tiles_m;

        // Operand sources.  Direct loads: a wave-uniform base pointer per wave instruction (scalar
        // registers, advanced by scalar adds) plus a 32-bit per-lane byte offset that never changes,
        // so that issuing a k-tile's loads costs no vector ALU work.  Staged loads: per-thread pointers.
        const uint16_t* wsrc[WPASS];
        const uint16_t* xsrc[XPASS];
        unsigned woff[WPASS], xoff[XPASS];
#pragma unroll
        for (int i = 0; i < WPASS; ++i) {
            const int blk = wv * WPASS + i;                          // (uniform) block of ROWS_PER_DMA rows
            const int v = W_DMA ? blk * ROWS_PER_DMA + lane / GPIECES : vr0 + ROWS_PER_PASS * i;
            const int piece = W_DMA ? slot ^ swz_f<GPIECES>(v) : vp;
            if (is_swiglu(EPI)) {
                const int j0 = tile_n * JPT;                         // first row of the tile: always valid
                int j = j0 + (v >> 4) * 8 + (v & 7);
                j = j < a.N ? j : a.N - 1;
                if (W_DMA && W_SBASE) {
                    // ROWS_PER_DMA = 8: a wave instruction covers 8 gate rows or the 8 matching up rows
                    wsrc[i] = ((blk & 1) ? a.w1 : a.w0) + (size_t)j0 * K;
                    woff[i] = (unsigned)((j - j0) * K + piece * 8) * 2u;
                } else {
                    wsrc[i] = (((v >> 3) & 1) ? a.w1 : a.w0) + (size_t)j * K + piece * 8;
                    woff[i] = 0;
                }
            } else {
                const int n0 = tile_n * BN;
                int n = n0 + v;
                n = n < a.N ? n : a.N - 1;
                if (W_DMA) {
                    wsrc[i] = a.w0 + (size_t)n0 * K;
                    woff[i] = (unsigned)((n - n0) * K + piece * 8) * 2u;
                } else {
                    wsrc[i] = a.w0 + (size_t)n * K + piece * 8;
                    woff[i] = 0;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < XPASS; ++i) {
            const int v = X_DMA ? (wv * XPASS + i) * ROWS_PER_DMA + lane / GPIECES : vr0 + ROWS_PER_PASS * i;
            const int piece = X_DMA ? slot ^ swz_f<GPIECES>(v) : vp;
            const int m0 = tile_m * BM;
            int m = m0 + v;
            m = m < a.M ? m : a.M - 1;       // rows past M are loaded from a valid row and never stored
            if (X_DMA) {
                xsrc[i] = a.x + (size_t)m0 * K;
                xoff[i] = (unsigned)((m - m0) * K + piece * 8) * 2u;
            } else {
                xsrc[i] = a.x + (size_t)m * K + piece * 8;
                xoff[i] = 0;
            }
        }

        uintx4 wreg[W_DMA ? 1 : WPASS], xreg[X_DMA ? 1 : XPASS];

        // K is a multiple of 8, so a 16-byte piece is entirely inside or outside [0,K); with KTAIL the
        // pieces past K are read from the row start (valid memory) and replaced by zeros.
        auto load_w = [&](int kt, int buf) {      // DMA: lands in stage buf; else: into wreg
#pragma unroll
            for (int i = 0; i < WPASS; ++i) {
                if (W_DMA && W_SBASE) {
                    dma16_sbase(wsrc[i] + kt * GK, woff[i], smem + buf * STAGE + (wv * WPASS + i) * 64);
                } else if (W_DMA) {
                    dma16(wsrc[i] + kt * GK, smem + buf * STAGE + (wv * WPASS + i) * 64);
                } else {
                    const bool kok = kt * GK + vp * 8 < K;
                    uintx4 v = *reinterpret_cast<const uintx4*>(wsrc[i] + (kok ? kt * GK : -vp * 8));
                    wreg[i] = kok ? v : zero4;
                }
            }
        };
        auto load_x = [&](int kt, int buf) {
#pragma unroll
            for (int i = 0; i < XPASS; ++i) {
                if (X_DMA) {
                    dma16_sbase(xsrc[i] + kt * GK, xoff[i], smem + buf * STAGE + BN * GPIECES + (wv * XPASS + i) * 64);
                } else {
                    const bool kok = !KTAIL || kt * GK + vp * 8 < K;
                    uintx4 v = *reinterpret_cast<const uintx4*>(xsrc[i] + (kok ? kt * GK : -vp * 8));
                    xreg[i] = kok ? v : zero4;
                }
            }
        };
        auto store_w = [&](int buf) {             // VGPR path only
            if (!W_DMA) {
#pragma unroll
                for (int i = 0; i < WPASS; ++i) smem[buf * STAGE + swz<GPIECES>(vr0 + ROWS_PER_PASS * i, vp)] = wreg[i];
            }
        };
        auto store_x = [&](int buf) {
            if (!X_DMA) {
#pragma unroll
                for (int i = 0; i < XPASS; ++i) {
                    smem[buf * STAGE + BN * GPIECES + swz<GPIECES>(vr0 + ROWS_PER_PASS * i, vp)] = xreg[i];
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

        half8 wa[2][TN], xb[2][TM];
        auto frags = [&](int buf, int kk, int fs) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                wa[fs][tn] = __builtin_bit_cast(half8, smem[buf * STAGE + swz<GPIECES>(wn * (BN / WN) + tn * 32 + lr, 2 * kk + lg)]);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                xb[fs][tm] = __builtin_bit_cast(half8, smem[buf * STAGE + BN * GPIECES + swz<GPIECES>(wm * (BM / WM) + tm * 32 + lr, 2 * kk + lg)]);
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

        // ---- prologue: the first NS k-tiles into the NS stages; VGPR-path operands run one tile further
        const int nk = ke - kb;
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            if (st < nk) {
                load_w(kb + st, st); load_x(kb + st, st);
                store_w(st); store_x(st);
            }
        }
        if (nk > NS) {
            if (!W_DMA) load_w(kb + NS, 0);
            if (!X_DMA) load_x(kb + NS, 0);
        }
        if (W_DMA || X_DMA) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();

        constexpr int LPT = (W_DMA ? WPASS : 0) + (X_DMA ? XPASS : 0);   // direct loads per k-tile per wave
        if constexpr (FD == 2) {
            static_assert(NS == 2 && KSTEPS == 4 && W_DMA && X_DMA, "three fragment buffers: two stages of four k-steps, direct loads");
            half8 wa3[3][TN], xb3[3][TM];
            auto frags3 = [&](int buf, int kk, int fs) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    wa3[fs][tn] = __builtin_bit_cast(half8, smem[buf * STAGE + swz<GPIECES>(wn * (BN / WN) + tn * 32 + lr, 2 * kk + lg)]);
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    xb3[fs][tm] = __builtin_bit_cast(half8, smem[buf * STAGE + BN * GPIECES + swz<GPIECES>(wm * (BM / WM) + tm * 32 + lr, 2 * kk + lg)]);
            };
            auto mfmas3 = [&](int fs) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
                        acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wa3[fs][tn], xb3[fs][tm], acc[tn][tm], 0, 0, 0);
            };
            frags3(0, 0, 0);
            frags3(0, 1, 1);
            // k-step s of k-tile `it` is global step 4 it + s and lives in fragment buffer (it + s) mod 3; while it is
            // multiplied, step + 2 is read.  The barrier sits in the middle of the k-tile: all four k-steps of
            // stage st have been read by then, k-tile it+1 must have landed, and its first fragments are read
            // right behind it.  (A k-tile that does not exist is "read" from the current stage and never used.)
            auto tile = [&](auto ph, int it) __attribute__((always_inline)) {
                constexpr int P = decltype(ph)::value;
                const int st = it % NS;
                const int nx = (it + 1 < nk) ? (it + 1) % NS : st;
                frags3(st, 2, (P + 2) % 3); mfmas3(P % 3); interleave();
                frags3(st, 3, (P + 3) % 3); mfmas3((P + 1) % 3); interleave();
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
                if (it + NS < nk) { load_w(kb + it + NS, st); load_x(kb + it + NS, st); }
                frags3(nx, 0, (P + 4) % 3); mfmas3((P + 2) % 3); interleave();
                frags3(nx, 1, (P + 5) % 3); mfmas3((P + 3) % 3); interleave();
            };
            for (int it = 0; it < nk; it += 3) {
                tile(std::integral_constant<int, 0>{}, it);
                if (it + 1 < nk) tile(std::integral_constant<int, 1>{}, it + 1);
                if (it + 2 < nk) tile(std::integral_constant<int, 2>{}, it + 2);
            }
        } else {
        frags(0, 0, 0);
        for (int it = 0; it < nk; ++it) {
            const int st = it % NS;
#pragma unroll
            for (int kk = 0; kk < KSTEPS - 1; ++kk) {
                frags(st, kk + 1, (kk + 1) & 1);
                mfmas(kk & 1);
                interleave();
            }
            // Every read of stage st has been issued.  Before the barrier, k-tile it+1 must have landed:
            // direct loads complete in order, so it is enough that at most the loads of the k-tiles
            // behind it (up to NS-2 of them) are still in flight.  The compiler does not carry these
            // loads across the loop edge, hence the explicit wait.
            if (LPT > 0) {
                int behind = nk - 2 - it;            // k-tiles after it+1 that have been requested
                behind = behind < NS - 2 ? behind : NS - 2;
                static_assert((NS - 2) * LPT < 64, "wait count out of range");
                if (behind <= 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                else if (behind == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPT) : "memory");
                else if (behind == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NS > 3 ? 2 * LPT : 0) : "memory");
                else if (behind == 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NS > 4 ? 3 * LPT : 0) : "memory");
                else if (behind == 4) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NS > 5 ? 4 * LPT : 0) : "memory");
                else if (behind == 5) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NS > 6 ? 5 * LPT : 0) : "memory");
                else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NS > 7 ? 6 * LPT : 0) : "memory");
            }
            __syncthreads();
            if (it + NS < nk) {
                if (W_DMA) load_w(kb + it + NS, st); else store_w(st);
                if (X_DMA) load_x(kb + it + NS, st); else store_x(st);
                if (it + NS + 1 < nk) {
                    if (!W_DMA) load_w(kb + it + NS + 1, st);
                    if (!X_DMA) load_x(kb + it + NS + 1, st);
                }
            }
            if (it + 1 < nk) frags((it + 1) % NS, 0, 0);
            mfmas((KSTEPS - 1) & 1);
        }
        }

        // ---- whole tile: finished below; shared tile: leave the fp32 partial for the fix-up kernel ---
        const bool whole = (kb == 0 && ke == ktiles);
        if (!whole) {
            const int pslot = (t == first_tile) ? 0 : 1;
            floatx4* ps = reinterpret_cast<floatx4*>(a.partials + ((size_t)worker * 2 + pslot) * (BN * BM));
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        ps[((tn * TM + tm) * 4 + q) * THREADS + tid] =
                            floatx4{acc[tn][tm][4 * q], acc[tn][tm][4 * q + 1], acc[tn][tm][4 * q + 2], acc[tn][tm][4 * q + 3]};
        }

        // ---- epilogue ------------------------------------------------------------------------
        if (whole) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    store_fragment<BN, BM, WN, WM, EPI>(a, tile_n, tile_m, wn, wm, tn, tm, lr, lg, acc[tn][tm]);
        }
        // the next run rewrites the LDS stages only after this barrier
        __syncthreads();
    }
}

// Time model (microseconds) of running `tiles` tiles of BN x BM on `grid` workgroups.
//   whole tiles only : ceil(tiles / grid) rounds;
//   shared remainder : floor(tiles / grid) whole rounds; the ragged remainder is cut along K and a second
//                      pass (one more launch, the partial tiles' round trip through memory) adds the parts.
// How the remainder is cut depends on what bounds the kernel.  With several token tiles it is the matrix
// cores, fed through the L2: workgroups on neighbouring tiles must walk the same k range at the same
// time or the panels they share are fetched once per workgroup (measured: a 30B-shaped down projection,
// 208 tiles of 256x256 on 256 workgroups in equal contiguous shares, ran HBM-bound at 585 us against 485
// us for whole tiles on 208 workgroups).  So every remainder tile is cut into the same `parts` = grid /
// remainder equal k ranges (whole tiles if that is 1) -- also with a single token tile of 256, whose
// activation panel is shared by every workgroup and too large for an L2 (measured on the 30B-shaped down
// projection at M = 256: 88 us against 97-113 us with contiguous shares), unless equal ranges would leave
// more than a tenth of the workgroups idle (7B-shaped gate/up at M = 160: 86 tiles x 2 ranges on 256
// workgroups, 81 against 75 us; 13B-shaped, 108 tiles x 2: 106 against 97 us).  The few-token configurations (one token tile of at most 128) are bound
// by their weight traffic, every weight panel is read exactly once whatever the cut, and equal contiguous
// shares (parts = 0) keep every workgroup busy.
// A workgroup's speed by configuration, fitted to measurements of every configuration and cut on the four
// projections of the 7B..70B shapes at M = 256..2048 (weight copies rotated so that they come from HBM;
// clocks settled under each shape's load for 40 ms first -- after a lighter kernel the first launches run
// up to 15 % slower): 256x256 tiles 4.7 TFLOP/s + 6 us per tile, 128x128 tiles two per CU 1.8 TFLOP/s + 6
// us, 128x128 with three stages one per CU 3.4 TFLOP/s + 4 us; the second pass 5 us + its bytes at ~8
// TB/s (they are still in the caches).  On those 64 shapes the pick is on average 0.5 % slower than the
// best of the six (configuration, cut) pairs, 8 % at worst.
struct Schedule {
    int sk_tiles;      // tiles cut along K (0: whole tiles only)
    int parts;         // equal k ranges per shared tile; 0 = equal contiguous shares across tile boundaries
    double us;
};

Schedule plan_schedule(int tiles, int tiles_m, int grid, int BN, int BM, int K, double wg_tflops, double tile_fixed_us)
{
    double work_us = 2.0 * BN * BM * (double)K / (wg_tflops * 1e6);
    if (tiles_m == 1) {      // every weight panel is read by one workgroup only: its traffic is a second bound
        const double stream_us = (double)BN * K * 2.0 / (6.0e6 / grid);
        work_us = work_us > stream_us ? work_us : stream_us;
    }
    const double tile_us = tile_fixed_us + work_us;
    const int rem = tiles % grid, full = tiles / grid;
    const double tile_bytes = (double)BN * BM * 4.0;
    const double whole = (double)((tiles + grid - 1) / grid) * tile_us;
    if (rem == 0) return Schedule{0, tiles_m == 1 ? 0 : 1, whole};
    const int ktiles = (K + 63) / 64;
    int parts = grid / rem;
    if (parts > ktiles) parts = ktiles;
    // One token tile: equal contiguous shares for the few-token configurations, and for a 256-token tile
    // when equal ranges would leave more than a tenth of the workgroups idle.
    if (tiles_m == 1 && (BM <= 128 || (long)rem * parts * 10 < (long)grid * 9)) {
        const double shared = ((double)full + (double)rem / grid) * tile_us + 5.0 + (double)(grid + rem) * tile_bytes * 2.0 / 4.0e6;
        return shared < whole ? Schedule{rem, 0, shared} : Schedule{0, 0, whole};
    }
    if (parts < 2) return Schedule{0, 1, whole};
    const double shared = (double)full * tile_us + tile_fixed_us + work_us / parts + 5.0 +
                          (double)rem * parts * tile_bytes * 2.0 / 8.0e6;
    return shared < whole ? Schedule{rem, parts, shared} : Schedule{0, 1, whole};
}

// the three multi-token-tile configurations
constexpr double BIG_TFLOPS = 4.7, BIG_FIXED_US = 6.0;        // 256x256, one workgroup per CU
constexpr double SMALL_TFLOPS = 1.8, SMALL_FIXED_US = 6.0;    // 128x128, two per CU
constexpr double DEEP_TFLOPS = 3.4, DEEP_FIXED_US = 4.0;      // 128x128, three stages, one per CU
constexpr double FEW_TFLOPS = 900.0 / 256;                    // one token tile: bound by the weight stream anyway

// ALL = also build the variant for a ragged K (operands staged through VGPRs); the direct-to-LDS
// configurations leave it to the 128x128 one.
template <int BN, int BM, int WN, int WM, int GK, int NS, bool ALL, int FD = 1>
hipError_t launch_cfg(GemmArgs a, int epilogue, int grid_cap, hipStream_t stream, double wg_tflops, double tile_fixed_us)
{
    const int per_tile = is_swiglu(epilogue) ? BN / 2 : BN;
    const int tiles_n = (a.N + per_tile - 1) / per_tile;
    const int tiles_m = (a.M + BM - 1) / BM;
    const int ktiles = (a.K + GK - 1) / GK;
    a.tiles = tiles_n * tiles_m;
    const long U = (long)a.tiles * ktiles;
    long grid = grid_cap;
    if (grid > U) grid = U;
    const Schedule plan = plan_schedule(a.tiles, tiles_m, (int)grid, BN, BM, a.K, wg_tflops, tile_fixed_us);
    const int sk_tiles = plan.sk_tiles, parts = plan.parts;
    const size_t lds = (size_t)NS * (BN + BM) * (GK / 8) * sizeof(uintx4);
    dim3 g((unsigned)grid), b(64 * WN * WM);
#define THI_LAUNCH_K(E, KT)                                                                                  \
    do {                                                                                                     \
        auto kern = gemm_streamk<BN, BM, WN, WM, GK, NS, E, KT, FD>;                                                  \
        static std::once_flag attr_once;      /* one opt-in per kernel variant, safe from several threads */  \
        std::call_once(attr_once, [&] {                                                                      \
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                   \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                 \
        });                                                                                                  \
        hipLaunchKernelGGL(kern, g, b, lds, stream, a, tiles_m, ktiles, sk_tiles, parts);                    \
        if (sk_tiles > 0)                                                                                    \
            hipLaunchKernelGGL((gemm_fixup<BN, BM, WN, WM, E>), dim3(2 * sk_tiles * (BN / WN / 32) * (BM / WM / 32)), \
                               b, 0, stream, a, tiles_m, ktiles, sk_tiles, (int)grid, parts);                \
    } while (0)
#define THI_LAUNCH(E)                                                                                        \
    do {                                                                                                     \
        if constexpr (ALL) {                                                                                 \
            if (a.K % GK) THI_LAUNCH_K(E, true);                                                             \
            else THI_LAUNCH_K(E, false);                                                                     \
        } else {                                                                                             \
            THI_LAUNCH_K(E, false);                                                                          \
        }                                                                                                    \
    } while (0)
    switch (epilogue) {
    case EPI_PLAIN: THI_LAUNCH(EPI_PLAIN); break;
    case EPI_ROPE: THI_LAUNCH(EPI_ROPE); break;
    case EPI_RMSNORM:            // RMSNorm runs as a pass of its own in front of the GEMM: the dispatcher
    case EPI_RMSNORM_ROPE:       // calls this with the plain / rotary / SwiGLU kinds only
    case EPI_RMSNORM_SWIGLU:
        return hipErrorInvalidValue;
    default: THI_LAUNCH(EPI_SWIGLU); break;
    }
#undef THI_LAUNCH
#undef THI_LAUNCH_K
    return hipGetLastError();
}

double config_cost(const GemmArgs& a, int epilogue, int BN, int BM, int grid, double wg_tflops, double tile_fixed_us)
{
    const int per_tile = is_swiglu(epilogue) ? BN / 2 : BN;
    const int tiles_m = (a.M + BM - 1) / BM;
    const long tiles = (long)((a.N + per_tile - 1) / per_tile) * tiles_m;
    const long units = tiles * ((a.K + 63) / 64);
    const int g = (int)(units < grid ? units : grid);
    return plan_schedule((int)tiles, tiles_m, g, BN, BM, a.K, wg_tflops, tile_fixed_us).us;
}

}  // namespace

namespace {

// One workgroup per token row: sum of squares in fp32, then the normalised row in fp16 (one rounding of
// x * r * gamma).  A memory-bound pass over M*K elements, a few percent of the GEMM it feeds.
__global__ __launch_bounds__(256) void rmsnorm_rows(const uint16_t* x, const uint16_t* gamma, float eps, uint16_t* xn, int K,
                                                    RopeArgs rope)
{
    // the rotary epilogue's table for this token: fp32 angle, full-range sincosf (positions reach
    // thousands of radians); done here so that the GEMM's epilogue needs neither
    if (rope.cs && (int)threadIdx.x < (rope.head_dim >> 1)) {
        float sn, cs;
        sincosf((float)rope.pos[blockIdx.x] * rope.theta[threadIdx.x], &sn, &cs);
        float* e = const_cast<float*>(rope.cs) + ((size_t)blockIdx.x * (rope.head_dim >> 1) + threadIdx.x) * 2;
        e[0] = cs;
        e[1] = sn;
    }
    __shared__ float s_part[4];
    const uint16_t* row = x + (size_t)blockIdx.x * K;
    uint16_t* dst = xn + (size_t)blockIdx.x * K;
    float ss = 0.f;
    for (int k = threadIdx.x * 8; k < K; k += 256 * 8) {
        const half8 v = __builtin_bit_cast(half8, *reinterpret_cast<const uintx4*>(row + k));
#pragma unroll
        for (int e = 0; e < 8; ++e) { const float f = (float)v[e]; ss = __builtin_fmaf(f, f, ss); }
    }
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) ss += __shfl_xor(ss, sh);
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float r = 1.0f / __builtin_sqrtf(((s_part[0] + s_part[1]) + (s_part[2] + s_part[3])) / (float)K + eps);
    for (int k = threadIdx.x * 8; k < K; k += 256 * 8) {
        const half8 v = __builtin_bit_cast(half8, *reinterpret_cast<const uintx4*>(row + k));
        const half8 g = __builtin_bit_cast(half8, *reinterpret_cast<const uintx4*>(gamma + k));
        half8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (_Float16)((float)v[e] * r * (float)g[e]);
        *reinterpret_cast<uintx4*>(dst + k) = __builtin_bit_cast(uintx4, o);
    }
}

}  // namespace

hipError_t launch_rmsnorm_rows(const uint16_t* x, const uint16_t* gamma, float eps, uint16_t* xn, int M, int K,
                               const RopeArgs& rope, hipStream_t stream)
{
    if (rope.cs && rope.head_dim > 2 * 256) return hipErrorInvalidValue;     // one thread per pair of the head
    hipLaunchKernelGGL(rmsnorm_rows, dim3((unsigned)M), dim3(256), 0, stream, x, gamma, eps, xn, K, rope);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& a, int epilogue, int num_cus, hipStream_t stream)
{
    int g_big = num_cus, g_small = 2 * num_cus;        // workgroups that fit: one resp. two per CU
    if (g_big * 4 > GEMM_MAX_GRID) g_big = GEMM_MAX_GRID / 4;
    if (g_small > GEMM_MAX_GRID) g_small = GEMM_MAX_GRID;
    // the direct-to-LDS configurations: plain / SwiGLU epilogues, K a multiple of the staged k-tile
    const bool direct = !is_rms(epilogue) && (a.K % 64 == 0);
    if (direct && a.M <= 128) {
        // Few tokens: one token tile, the weights are read once and the kernel is bound by how many
        // bytes a CU keeps in flight: three stages of 128 rows x 128 k against 64 tokens (K a multiple of
        // 128), else of 128 rows x 64 k against 128 tokens.  Every tile is cut along K here (far fewer
        // tiles than workgroups) and the second pass costs by the partial tiles' bytes, (workgroups +
        // tiles) x tile size: 128-row tiles halve them against 256-row tiles (7B-shaped O projection at
        // M = 128: 24.8 -> 18.5 us, gate/up 61 -> 53; second pass alone 8.5-9.7 us with 256 rows).  With
        // many more tiles than workgroups (70B-shaped gate/up: 448) the 256-row tile's smaller share of
        // activation staging wins instead (188 against 230 us).
        if (a.M <= 64 && a.K % 128 == 0) return launch_cfg<128, 64, 4, 1, 128, 3, false>(a, epilogue, g_big, stream, FEW_TFLOPS, 0.0);
        const int per_tile = is_swiglu(epilogue) ? 64 : 128;
        if ((a.N + per_tile - 1) / per_tile <= num_cus + num_cus / 8)
            return launch_cfg<128, 128, 2, 2, 64, 3, false>(a, epilogue, g_big, stream, FEW_TFLOPS, 0.0);
        return launch_cfg<256, 128, 4, 1, 64, 3, false>(a, epilogue, g_big, stream, FEW_TFLOPS, 0.0);
    }
    // 129..256 tokens and about as many 128-row tiles as workgroups (0.65..1.2 x: the gate/up shapes):
    // one token tile of 256 against 128 rows, so that the weights are read once and few tiles are cut
    // (7B-shaped gate/up at M = 192: 74.9 -> 67.4 us, 13B 98.9 -> 94.2, 30B 161 -> 152).  With fewer tiles
    // the 128 KiB partial tiles of the workgroups that share one cost more than reading the weights twice
    // (7B-shaped O projection 22.5 -> 31 us), with more the 256-row tile wins: both stay with the rule below.
    if (direct && a.M <= 256) {
        const int per_tile = is_swiglu(epilogue) ? 64 : 128;
        const long t128 = (a.N + per_tile - 1) / per_tile;
        if (t128 * 20 >= (long)num_cus * 13 && t128 * 5 <= (long)num_cus * 6)
            return launch_cfg<128, 256, 2, 4, 64, 3, false>(a, epilogue, g_big, stream, FEW_TFLOPS, 0.0);
    }
    // Several token tiles: the configuration with the smallest modelled time.  The three-stage 128x128
    // configuration runs one workgroup per CU, which only pays where the two-per-CU one would not have a
    // second workgroup for most CUs anyway (at most one 128x128 tile per CU).
    const double c_small = config_cost(a, epilogue, 128, 128, g_small, SMALL_TFLOPS, SMALL_FIXED_US);
    if (direct) {
        const double c_big = config_cost(a, epilogue, 256, 256, g_big, BIG_TFLOPS, BIG_FIXED_US);
        const int per_tile = is_swiglu(epilogue) ? 64 : 128;
        const long t128 = (long)((a.N + per_tile - 1) / per_tile) * ((a.M + 127) / 128);
        if (t128 <= num_cus) {
            const double c_deep = config_cost(a, epilogue, 128, 128, num_cus, DEEP_TFLOPS, DEEP_FIXED_US);
            if (c_deep < c_big && c_deep < c_small)
                return launch_cfg<128, 128, 2, 2, 64, 3, false>(a, epilogue, num_cus, stream, DEEP_TFLOPS, DEEP_FIXED_US);
        }
        if (c_big <= c_small) return launch_cfg<256, 256, 4, 2, 64, 2, false, 2>(a, epilogue, g_big, stream, BIG_TFLOPS, BIG_FIXED_US);
    }
    return launch_cfg<128, 128, 2, 2, 64, 2, true>(a, epilogue, g_small, stream, SMALL_TFLOPS, SMALL_FIXED_US);
}

}  // namespace thi
