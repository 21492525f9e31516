// Internal declarations shared by the translation units of libthi (never installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace thi {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

// What is fused around the linear operator.  RMSNORM*: x*gamma in front, the 1/rms scale behind.
// *SWIGLU: gate and up rows interleaved, silu(g)*u behind.  The plain and RMSNorm kinds add a residual
// behind the product when the argument block carries one.
// EPI_ROPE (GEMM only): the rotary epilogue on activations that were normalised by a pass of their own.
enum Epilogue { EPI_PLAIN = 0, EPI_RMSNORM = 1, EPI_SWIGLU = 2, EPI_RMSNORM_ROPE = 3, EPI_RMSNORM_SWIGLU = 4, EPI_ROPE = 5 };
constexpr bool is_rms(int epi) { return epi == EPI_RMSNORM || epi == EPI_RMSNORM_ROPE || epi == EPI_RMSNORM_SWIGLU; }
constexpr bool is_swiglu(int epi) { return epi == EPI_SWIGLU || epi == EPI_RMSNORM_SWIGLU; }
constexpr bool has_rope(int epi) { return epi == EPI_RMSNORM_ROPE || epi == EPI_ROPE; }

// Rotary embedding applied in the epilogue (EPI_RMSNORM_ROPE): interleaved pairs (2i, 2i+1) of every
// head in columns [0, n_rot); angle = pos[m] * theta[i].
struct RopeArgs {
    const int* pos;          // [M] token positions
    const float* theta;      // [head_dim / 2]
    int n_rot, head_dim;
    const float* cs;         // GEMM path: [M][head_dim / 2][2] = (cos, sin) of pos[m] * theta[i], made by the
                             // RMSNorm pass in front of the GEMM; nullptr in the decode kernels
};
constexpr int ROPE_TABLE_MAX_HEAD_DIM = 256;     // what the workspace reserves per token for that table

// ---- workspace layout (bytes from the workspace base) ----------------------
// [0, 64 KiB)             : status words (uint32), zero between calls: the stream-K decode kernel's
//                           hand-over flags (one per workgroup), the shared row blocks' arrival counters
//                           (one per block); last word: time-out marker
// [.., + hand-over bytes) : decode kernels: one hand-over slot per workgroup
// [.., + partial bytes)   : prefill GEMM: per-workgroup partial accumulator tiles (fp32)
// [.., + M*I*2)           : h = silu(gate)*up of the MLP (fp16)
// [.., + M*K*2)           : the normalised activations of the RMSNorm-fronted operators (prefill), then
//                           the rotary table of the QKV operator
constexpr size_t WS_COUNTER_BYTES = 64 * 1024;
constexpr int WS_MAX_COUNTERS = (int)(WS_COUNTER_BYTES / 4);

// ---- skinny (decode) kernel geometry ---------------------------------------
constexpr int SK_THREADS = 512;     // 8 waves
constexpr int SK_WAVES = 8;
constexpr int SK_ROWS = 128;        // virtual weight rows per tile (16 per wave)
constexpr int SK_KC = 256;          // k extent of one work unit
constexpr int SK_MAX_GRID = 512;    // upper bound on workgroups (sizes the hand-over slots)
constexpr int SK_MAX_MT = 4;        // token tiles of 16 per launch of the stream-K kernel (64 tokens)
constexpr unsigned SK_SPIN_LIMIT = 1u << 24;   // polls of a contributor's flag before a workgroup gives up
// hand-over slot of one workgroup: its partial tile (8 waves x up to 4 token tiles x 64 lanes x 4
// registers, fp32 bit patterns), then up to 64 partial sums of squares
constexpr int SK_SLOT_SSQ = SK_WAVES * SK_MAX_MT * 4 * 64;
constexpr int SK_SLOT_WORDS = SK_SLOT_SSQ + 16 * SK_MAX_MT;

struct SkinnyArgs {
    const uint16_t* x;       // [M,K] activations
    const uint16_t* gamma;   // [K] (RMSNorm) or nullptr
    const uint16_t* w0;      // weights [N,K]  (gate weights for SwiGLU)
    const uint16_t* w1;      // up weights [I,K] for SwiGLU, else nullptr
    uint16_t* out;           // [M,ldo]
    const uint16_t* residual; // [M,ldo] added behind the product (plain / RMSNorm kinds), or nullptr
    unsigned* handover;      // [grid][SK_SLOT_WORDS] hand-over slots
    unsigned* counters;      // [grid] hand-over flags, zero between calls; last word: time-out marker
    int M, N, K, ldo;        // N = physical rows of w0 (I for SwiGLU); ldo = out row length
    int tiles, kchunks;      // tiles of SK_ROWS virtual rows; chunks of SK_KC along K
    float eps;
    RopeArgs rope;
    unsigned spin_limit;     // stream-K: polls of a contributor's flag before the finishing workgroup gives up
    int withhold_flags;      // stream-K, test hook: contributors do not raise their flags (forces the give-up)
};

size_t skinny_handover_bytes();
hipError_t launch_skinny(const SkinnyArgs& a, int epilogue, int num_cus, hipStream_t stream);
// Row-slab decode kernel: a.tiles = slabs of 16 virtual rows; needs 1024 <= K <= ROWSLAB_MAX_K (a
// wave's slice of gamma must fit its share of LDS); uses no workspace.
constexpr int ROWSLAB_MAX_K = 32768;
hipError_t launch_rowslab(const SkinnyArgs& a, int epilogue, int num_cus, hipStream_t stream);
// Row-block decode kernel: the outputs dealt to the workgroups in equal contiguous blocks, T slabs of a
// block in flight at a time (same limits on K; a.tiles is not used; no workspace unless ksplit > 1).
struct RowBlockPlan {
    int per_wg;      // outputs (rows of W, gate/up pairs for SwiGLU) per workgroup
    int grid;        // workgroups
    int tiles;       // 16-row tiles per block
    int passes;      // passes over K
    int T;           // tiles in flight per pass (2..6)
    int ksplit;      // workgroups that share a block, each with 1/ksplit of K (1: nothing is handed over)
};
// ksplit > 1 (plain kind, one pass): blocks of ksplit x as many rows, so that a wave's slice of x serves
// ksplit x as many tiles; the block's workgroups hand their sums in through the stream-K kernel's
// hand-over slots (a.handover, a.counters) and the last to arrive adds them in share order.
constexpr int ROWBLOCK_MAX_SPLIT = 6;
RowBlockPlan plan_rowblock(int N, int epilogue, int num_cus, int ksplit = 1);
bool rowblock_split_ok(int N, int K, int epilogue, int num_cus, int ksplit);
hipError_t launch_rowblock(const SkinnyArgs& a, int epilogue, int num_cus, hipStream_t stream, int ksplit = 1);
// The decode MLP as one launch: gate/up row blocks (up: N = I, K = H, out = h), a grid-wide rendezvous on two status
// words, then the down projection's shared row blocks (down: x = h, N = H, K = I) with ksplit_down workgroups per block.
// status words of its rendezvous (the other users stay below 1024): the launch number on this workspace, then one
// tag word per workgroup; unlike all other status words these are not zero between calls
constexpr int MLP_EPOCH_WORD = 2047, MLP_FLAG_WORDS = 2048, MLP_MAX_GRID = 512;
bool mlp_fused_ok(int M, int H, int I, int epilogue_up, int num_cus, int ksplit_down);
hipError_t launch_mlp_fused(const SkinnyArgs& up, const SkinnyArgs& down, int epilogue_up, int num_cus, hipStream_t stream,
                            int ksplit_down);

// ---- GEMM (prefill) kernel ---------------------------------------------------
struct GemmArgs {
    const uint16_t* x;       // [M,K] (already normalised where RMSNorm sits in front)
    const uint16_t* w0;      // [N,K]
    const uint16_t* w1;      // up weights for SwiGLU
    uint16_t* out;           // [M,ldo]
    const uint16_t* residual; // [M,ldo] added behind the product (plain / RMSNorm kinds), or nullptr
    float* partials;         // [grid][2][tile] fp32 partial tiles of tiles that were cut along K
    int M, N, K, ldo;        // N = physical rows of w0
    int tiles;               // filled in by the launcher
    RopeArgs rope;
};
constexpr int GEMM_MAX_GRID = 2048;   // in units of 128x128 partial tiles (a 256x256 tile takes four)
size_t gemm_partial_bytes();
hipError_t launch_gemm(const GemmArgs& a, int epilogue, int num_cus, hipStream_t stream);
// xn[m,k] = fp16(x[m,k] * gamma[k] / sqrt(mean_k x[m,:]^2 + eps)): the prefill path's RMSNorm pass
// With rope.cs set it also fills that table: cs[m][i] = (cos, sin)(pos[m] * theta[i]), fp32, full-range.
hipError_t launch_rmsnorm_rows(const uint16_t* x, const uint16_t* gamma, float eps, uint16_t* xn, int M, int K,
                               const RopeArgs& rope, hipStream_t stream);

// ---- decode attention ---------------------------------------------------------
struct AttnArgs {
    const uint16_t* q;       // [B,Hq,D]
    const uint16_t* k;       // [B,Hkv,S_max,D]
    const uint16_t* v;       // [B,Hkv,S_max,D]
    const int* seq_lens;     // [B] live positions per request (device memory)
    uint16_t* out;           // [B,Hq,D]
    float* part;             // [B*Hq][nsplit][D + 2]: a chunk's unnormalised output, running maximum, running sum
    int B, Hq, Hkv, D, S_max;
    int group;               // Hq / Hkv query heads per cache head
    int chunk, nsplit;       // positions per chunk (a multiple of the kernel's quantum), chunks per request
    float scale2;            // softmax scale times log2(e)
};
constexpr int AT_MAX_SPLIT = 32;
int attention_heads_per_workgroup(int group);
int attention_chunk_quantum(int D, int gt);
hipError_t launch_attention(const AttnArgs& a, hipStream_t stream);

// Rotate one interleaved pair (a, b) = (y[c], y[c+1]), c even: Algorithm 1's  y*cos + mix*sin  with
// mix = (-b, a).  fp32 angle and full-range sinf/cosf (positions reach thousands of radians).
__device__ __forceinline__ void rope_pair(const RopeArgs& r, int m_pos, int c, float& a, float& b)
{
    if (c >= r.n_rot) return;
    const float ang = (float)m_pos * r.theta[(c % r.head_dim) >> 1];
    float sn, cs;
    sincosf(ang, &sn, &cs);
    const float na = a * cs - b * sn, nb = b * cs + a * sn;
    a = na;
    b = nb;
}

// The same rotation with cos and sin taken from the table in r.cs (token row m of this launch).
__device__ __forceinline__ void rope_pair_table(const RopeArgs& r, int m, int c, float& a, float& b)
{
    if (c >= r.n_rot) return;
    const float* e = r.cs + ((size_t)m * (r.head_dim >> 1) + ((c % r.head_dim) >> 1)) * 2;
    const float cs = e[0], sn = e[1];
    const float na = a * cs - b * sn, nb = b * cs + a * sn;
    a = na;
    b = nb;
}

// ---- small device helpers shared by the decode kernels -----------------------
constexpr int WT_STRIDE = 17;                  // 16-byte units per transposition row (256 B + 16 B pad)
constexpr int WT_UNITS = 16 * WT_STRIDE;       // per wave

__device__ __forceinline__ uintx4 ld_stream(const uint16_t* p) {      // weights: read once, keep out of the caches
    return __builtin_nontemporal_load(reinterpret_cast<const uintx4*>(p));
}
__device__ __forceinline__ uintx4 ld_cached(const uint16_t* p) {
    return *reinterpret_cast<const uintx4*>(p);
}
__device__ __forceinline__ float silu_mul(float g, float u) {
    return g / (1.0f + __expf(-g)) * u;
}
__device__ __forceinline__ float half_bits_to_float(uint16_t b) {
    return (float)__builtin_bit_cast(_Float16, b);
}
__device__ __forceinline__ uint16_t to_half_bits(float v) {
    _Float16 h = (_Float16)v;   // round-to-nearest-even
    return __builtin_bit_cast(uint16_t, h);
}

hipError_t launch_fill_words(void* ptr, size_t bytes, uint32_t value, hipStream_t stream);

}  // namespace thi
