// C-ABI entry points of libthi: argument validation, workspace carving and
// dispatch on M between the weight-streaming decode kernels and the MFMA GEMM.
// The declarations and their contract are in include/thi.h.
#include "../../include/thi.h"
#include "thi_internal.h"

#include <atomic>
#include <mutex>

namespace {

using namespace thi;

constexpr int THI_VERSION = 100;          // 0.1.0
constexpr int SKINNY_GROUP = 32;          // tokens per skinny launch
constexpr int SKINNY_MAX_M = 32;          // automatic dispatch: M <= this -> skinny kernels (measured crossover)

std::atomic<int> g_family{0};
std::atomic<int> g_rowblock_split{0};      // 0: chosen per call; >= 1: forced where the shape admits it
std::atomic<unsigned> g_spin_limit{SK_SPIN_LIMIT};   // polls of a hand-over flag before a workgroup gives up
std::atomic<int> g_withhold_flags{0};      // test hook: contributors never raise their flags
std::atomic<int> g_mlp_fusion{0};          // opt-in: the decode MLP as one launch where the fused kernel serves the shape

int device_cu_count()
{
    // once-initialised, per-device cache of the CU count (the only state the library keeps)
    static std::atomic<int> cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int v = cache[dev].load(std::memory_order_relaxed);
    if (v > 0) return v;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    cache[dev].store(cus, std::memory_order_relaxed);
    return cus;
}

inline bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Workspace {
    unsigned* counters;
    unsigned* handover;
    float* partials;  // GEMM kernels: partial accumulator tiles; nullptr when the workspace was sized for decode only
    uint16_t* h;     // MLP: silu(gate)*up [M,I]
    uint16_t* xn;    // prefill: normalised activations [M,K] of the RMSNorm-fronted operators (with the GEMM region only)
    float* rope_cs;  // prefill, QKV with the rotary epilogue: (cos, sin) table [M][head_dim/2][2], behind xn
};

// The decode kernels' part: status words, then the hand-over slots.  Decode attention puts its partial
// results behind it, so that a workspace shared with the other calls keeps its status words.
size_t fixed_bytes() { return WS_COUNTER_BYTES + round_up(skinny_handover_bytes(), 256); }

// The GEMM kernels run above SKINNY_MAX_M tokens (or when they are forced): only then does a workspace
// carry their partial-tile region and the normalised activations of the RMSNorm pass.
bool gemm_possible(int M) { return M > SKINNY_MAX_M || g_family.load(std::memory_order_relaxed) == 2; }

// (op, M, a, b) = (RMSNORM_QKV or LINEAR, M, N, K) or (SWIGLU_MLP, M, H, I); byte offsets from the base
struct Layout {
    size_t partials, h, xn, rope_cs, total;
};
Layout layout(int op, int M, int a, int b, bool gemm)
{
    Layout l;
    l.partials = fixed_bytes();
    l.h = l.partials + (gemm ? gemm_partial_bytes() : 0);
    l.xn = l.h + (op == THI_OP_SWIGLU_MLP ? round_up((size_t)M * (size_t)b * 2, 256) : 0);
    size_t xn = 0, cs = 0;
    if (gemm && op == THI_OP_RMSNORM_QKV) {      // [M,K], then the rotary table [M][<= 128][2] fp32
        xn = round_up((size_t)M * (size_t)b * 2, 256);
        cs = (size_t)M * (ROPE_TABLE_MAX_HEAD_DIM / 2) * 8;
    } else if (gemm && op == THI_OP_SWIGLU_MLP) {
        xn = round_up((size_t)M * (size_t)a * 2, 256);      // [M,H]
    }
    l.rope_cs = l.xn + xn;
    l.total = l.rope_cs + cs;
    return l;
}

size_t workspace_need(int op, int M, int a, int b) { return layout(op, M, a, b, gemm_possible(M)).total; }

// A workspace large enough for the GEMM layout is carved that way (so one sized while the GEMM kernels were
// forced keeps working afterwards); a smaller one holds the decode layout.
Workspace carve(void* base, size_t bytes, int op, int M, int a, int b)
{
    const Layout with = layout(op, M, a, b, true);
    const bool gemm = bytes >= with.total;
    const Layout l = gemm ? with : layout(op, M, a, b, false);
    char* p = static_cast<char*>(base);
    Workspace w;
    w.counters = reinterpret_cast<unsigned*>(p);
    w.handover = reinterpret_cast<unsigned*>(p + WS_COUNTER_BYTES);
    w.partials = gemm ? reinterpret_cast<float*>(p + l.partials) : nullptr;
    w.h = reinterpret_cast<uint16_t*>(p + l.h);
    w.xn = reinterpret_cast<uint16_t*>(p + l.xn);
    w.rope_cs = reinterpret_cast<float*>(p + l.rope_cs);
    return w;
}

// Row blocks, modelled time in microseconds with `split` workgroups per block (the constants are
// explained with the other two kernels' above pick_decode_kernel)
double rowblock_time(int M, int N, int K, int epilogue, int cus, int split)
{
    const bool swiglu = is_swiglu(epilogue);
    const int out_per_tile = swiglu ? 8 : 16;
    const double t_w = (swiglu ? 2.0 : 1.0) * (double)N * (double)K * 2.0 / 7.0e6;
    const int groups = (K + 127) / 128, groups_max = (groups + 8 * split - 1) / (8 * split), units_max = (groups_max + 1) / 2;
    double ragged = (double)units_max * SK_KC * SK_WAVES * split / (double)K;
    if (ragged < 1.0) ragged = 1.0;
    const RowBlockPlan bp = plan_rowblock(N, epilogue, cus, split);
    const double per_pass = (double)bp.per_wg / out_per_tile / bp.passes;      // tiles sharing one load of x
    const double x_extra = (M <= 4 ? 0.0 : M <= 8 ? 0.05 : M <= 16 ? 0.15 : 0.40) / per_pass;
    const double lacking = (double)bp.per_wg * (cus / split) / (double)N;
    // plain kind: the rows a block's last tile lacks still cost their load instructions
    const double fill = epilogue == EPI_PLAIN ? (double)bp.tiles * out_per_tile / (double)bp.per_wg : 1.0;
    return 3.8 + 0.5 * (bp.passes - 1) + ((split == 1 && bp.tiles <= 2 && K >= 8192 && K < 16384) ? 4.0 : 0.0) +
           (split > 1 ? 1.75 + (bp.tiles <= 2 ? 1.0 : 0.0) : 0.0) +
           t_w * (1.0 + x_extra) * (1.0 + 0.2 * (ragged - 1.0)) * (1.0 + 0.5 * (fill - 1.0)) * lacking;
}

// Row blocks: how many workgroups share a block (1 = none)?  The smallest modelled time.  Not above
// K = 24576: the 70B down projection (K = 28672) measured 15 % slower with two workgroups on the halves
// of its 56 KiB rows than the model says.
int pick_rowblock_split(int M, int N, int K, int epilogue, int cus)
{
    const int forced = g_rowblock_split.load(std::memory_order_relaxed);
    if (forced >= 1) return rowblock_split_ok(N, K, epilogue, cus, forced) ? forced : 1;
    if (epilogue != EPI_PLAIN || K > 24576) return 1;
    int best = 1;
    double t_best = rowblock_time(M, N, K, epilogue, cus, 1);
    for (int s = 2; s <= 4; ++s) {
        if (!rowblock_split_ok(N, K, epilogue, cus, s)) continue;
        const double t = rowblock_time(M, N, K, epilogue, cus, s);
        if (t < t_best) { t_best = t; best = s; }
    }
    return best;
}

// Decode: which of the three weight-streaming kernels?
//   stream-K   : work units of 128 rows x 256 k in equal contiguous shares: perfect balance whatever the
//                shape, a hand-over between workgroups at the end;
//   row slabs  : slabs of 16 rows over the whole of K, dealt round-robin: no hand-over, but the slabs
//                must divide well among the compute units and every wave reads its slice of x per slab;
//   row blocks : N / #CUs rows per workgroup in one contiguous block, several 16-row tiles in flight
//                sharing the wave's slice of x: no hand-over, balanced whenever N >> #CUs.
// Decided by a time model in microseconds whose constants were fitted to measured (shape, M) points on
// MI355X (17 shapes: the 7B..70B projections and a 32000-row output head, M = 1..32; the pick is within
// 3 % of the best of the three on all but a handful, 5 % at worst).  t_w = weight bytes / 7.0 TB/s; a
// wave's last unit of 256 k may be partly empty (ragged, slabs and blocks).
//   stream-K   : ~5.5 us fixed + 1.06 t_w + the hand-over, 0.5 + 0.05 M us up to M = 16 and ~5 us above;
//   row slabs  : ~3.5 us fixed; slowed by the slots a ragged last round leaves empty, by the activation
//                traffic (x1.02 at M<=4, x1.09 at M<=8, x1.15 at M<=16, x1.45 above) and by ~10 % for
//                the RMSNorm prologue;
//   row blocks : ~3.8 us fixed (all tiles of a pass finish together: their reduction is not hidden),
//                0.5 us per further pass over K, 4 us more with one or two tiles per workgroup and
//                8192 <= K < 16384 (measured on the 70B O and 13B down projections); the activation
//                traffic is shared by the tiles of a pass (+5 % / +15 % / +40 % at M <= 8 / 16 / 32,
//                divided by the tiles per pass); a ragged last unit costs about a fifth of what it
//                costs the slabs; slowed by the rows the last workgroup lacks.  With S workgroups per
//                block (plain kind): S x the tiles share a load of x, the eight waves of S workgroups
//                divide K, and the hand-over at the end costs ~1.75 us (1 us more with one or two tiles
//                per block); plain kind: the rows that the block's last tile lacks cost half of what
//                rows with weights cost (20 rows in two tiles: +30 %).
enum DecodeKernel { DK_STREAMK = 1, DK_ROWSLAB = 3, DK_ROWBLOCK = 4 };
int pick_decode_kernel(int M, int N, int K, int epilogue, int cus)
{
    if (K < 1024 || K > ROWSLAB_MAX_K) return DK_STREAMK;
    const int fam = g_family.load(std::memory_order_relaxed);
    if (fam == 1) return DK_STREAMK;
    if (fam == 3) return DK_ROWSLAB;
    if (fam == 4) return DK_ROWBLOCK;
    const bool swiglu = is_swiglu(epilogue);
    const int out_per_tile = swiglu ? 8 : 16;
    const double t_w = (swiglu ? 2.0 : 1.0) * (double)N * (double)K * 2.0 / 7.0e6;
    const int groups = (K + 127) / 128, groups_max = (groups + 7) / 8, units_max = (groups_max + 1) / 2;
    double ragged = (double)units_max * SK_KC * SK_WAVES / (double)K;
    if (ragged < 1.0) ragged = 1.0;

    const double t_sk = 5.5 + 1.06 * t_w + (M <= 16 ? 0.5 + 0.05 * M : 5.0);

    const long slabs = ((long)N + out_per_tile - 1) / out_per_tile;
    const long rounds = (slabs + cus - 1) / cus;
    const double fill = (double)slabs / (double)(rounds * cus);
    const double x_slab = M <= 1 ? 1.0 : M <= 4 ? 1.02 : M <= 8 ? 1.09 : M <= 16 ? 1.15 : 1.45;
    const double t_slab = 3.5 + t_w * x_slab * ragged / fill * (is_rms(epilogue) ? 1.10 : 1.0);

    const double t_block = rowblock_time(M, N, K, epilogue, cus, pick_rowblock_split(M, N, K, epilogue, cus));

    if (t_block < t_slab && t_block < t_sk) return DK_ROWBLOCK;
    return t_slab < t_sk ? DK_ROWSLAB : DK_STREAMK;
}

// Which kernel runs a projection of M tokens, and how many tokens a launch takes.
//   M <= 32       : a decode kernel (pick_decode_kernel), one launch.
//   33 <= M <= 64 : the stream-K decode kernel takes up to 64 tokens per launch (its activations are
//                   shared by the workgroup's waves through LDS, so the wider batch costs it least); it
//                   runs where its modelled time beats the few-token GEMM's (fitted on the 7B..70B
//                   projections: stream-K 5.5 us + 1.06 t_w + 8 us with three token tiles / 13 us with
//                   four; GEMM 8 us for its two launches, 5 more for the RMSNorm pass, + 1.5 t_w up to
//                   t_w = 30 us and 1.25 t_w beyond).  Typically: everything but the smallest matrices up
//                   to 48 tokens, about a tie above.
//   M > 64        : the GEMM kernels.
// A forced family overrides this (forced stream-K: 64 tokens per launch; forced row slabs / blocks: 32).
struct DecodePlan {
    int kernel;     // DK_*, or 0 = the GEMM kernels
    int group;      // tokens per launch
};
DecodePlan plan_decode(int M, int N, int K, int epilogue, int cus)
{
    const int fam = g_family.load(std::memory_order_relaxed);
    if (fam == 2) return DecodePlan{0, 0};
    const int first = M < SKINNY_GROUP ? M : SKINNY_GROUP;
    if (fam == 1) return DecodePlan{DK_STREAMK, M > SKINNY_GROUP ? 16 * SK_MAX_MT : SKINNY_GROUP};
    if (fam == 3 || fam == 4) return DecodePlan{pick_decode_kernel(first, N, K, epilogue, cus), SKINNY_GROUP};
    if (M <= SKINNY_MAX_M) return DecodePlan{pick_decode_kernel(first, N, K, epilogue, cus), SKINNY_GROUP};
    if (M > 16 * SK_MAX_MT) return DecodePlan{0, 0};
    const double t_w = (is_swiglu(epilogue) ? 2.0 : 1.0) * (double)N * (double)K * 2.0 / 7.0e6;
    const double t_sk = 5.5 + 1.06 * t_w + (M <= 48 ? 8.0 : 13.0);
    const double t_gemm = (is_rms(epilogue) ? 13.0 : 8.0) + 1.5 * (t_w < 30.0 ? t_w : 30.0) + 1.25 * (t_w > 30.0 ? t_w - 30.0 : 0.0);
    if (t_sk < t_gemm) return DecodePlan{DK_STREAMK, 16 * SK_MAX_MT};
    return DecodePlan{0, 0};
}

// One fused projection: out[M, ldo] = epilogue( prologue(x)[M,K] * w^T ), any M.
int run_projection(const uint16_t* x, const uint16_t* gamma, float eps, const uint16_t* w0, const uint16_t* w1,
                   uint16_t* out, int M, int N, int K, int ldo, int epilogue, const Workspace& ws,
                   hipStream_t stream, RopeArgs rope = RopeArgs{nullptr, nullptr, 0, 2, nullptr},
                   const uint16_t* residual = nullptr)
{
    const int cus = device_cu_count();
    (void)hipGetLastError();      // an error another user of the runtime left behind is not ours to report
    const DecodePlan dp = plan_decode(M, N, K, epilogue, cus);
    if (dp.kernel != 0) {
        const int kernel = dp.kernel, group = dp.group;
        const bool slab = kernel != DK_STREAMK, block = kernel == DK_ROWBLOCK;
        const int rows_per_tile = slab ? (is_swiglu(epilogue) ? 8 : 16) : (is_swiglu(epilogue) ? SK_ROWS / 2 : SK_ROWS);
        const int tiles = (N + rows_per_tile - 1) / rows_per_tile;
        if ((long)tiles * ((K + SK_KC - 1) / SK_KC) > (1L << 30)) return THI_ERR_SHAPE;
        for (int m0 = 0; m0 < M; m0 += group) {
            SkinnyArgs a{};
            a.x = x + (size_t)m0 * K;
            a.gamma = gamma;
            a.w0 = w0;
            a.w1 = w1;
            a.out = out + (size_t)m0 * ldo;
            a.residual = residual ? residual + (size_t)m0 * ldo : nullptr;
            a.handover = ws.handover;
            a.counters = ws.counters;
            a.M = (M - m0 < group) ? M - m0 : group;
            a.N = N;
            a.K = K;
            a.ldo = ldo;
            a.tiles = tiles;
            a.kchunks = (K + SK_KC - 1) / SK_KC;
            a.eps = eps;
            a.rope = rope;
            a.spin_limit = g_spin_limit.load(std::memory_order_relaxed);
            a.withhold_flags = g_withhold_flags.load(std::memory_order_relaxed);
            if (rope.pos) a.rope.pos = rope.pos + m0;
            hipError_t e;
            if (!slab) e = launch_skinny(a, epilogue, cus, stream);
            else if (block) e = launch_rowblock(a, epilogue, cus, stream, pick_rowblock_split(a.M, N, K, epilogue, cus));
            else e = launch_rowslab(a, epilogue, cus, stream);
            if (e != hipSuccess) return THI_ERR_HIP;
        }
        return THI_OK;
    }
    if (!ws.partials) return THI_ERR_WORKSPACE;      // sized for the decode kernels only (see thi_workspace_bytes)
    {
        const long tn = (N + 63) / 64, tm = (M + 127) / 128;     // upper bound on tiles of any configuration
        if (tn * tm > WS_MAX_COUNTERS) return THI_ERR_SHAPE;
    }
    // Prefill: RMSNorm runs as a pass of its own (a few percent of the GEMM's time) so that the GEMM can
    // take both operands straight from memory into LDS in its fastest configuration; the decode kernels
    // keep it fused, where a second pass over x would cost a launch.
    if (is_rms(epilogue)) {
        RopeArgs table = rope;
        if (has_rope(epilogue)) {
            if (rope.head_dim > ROPE_TABLE_MAX_HEAD_DIM) return THI_ERR_SHAPE;
            table.cs = rope.cs = ws.rope_cs;
        }
        if (launch_rmsnorm_rows(x, gamma, eps, ws.xn, M, K, table, stream) != hipSuccess) return THI_ERR_HIP;
        x = ws.xn;
        gamma = nullptr;
        epilogue = epilogue == EPI_RMSNORM ? EPI_PLAIN : epilogue == EPI_RMSNORM_ROPE ? EPI_ROPE : EPI_SWIGLU;
    }
    GemmArgs g{};
    g.x = x;
    g.w0 = w0;
    g.w1 = w1;
    g.out = out;
    g.residual = residual;
    g.partials = ws.partials;
    g.tiles = 0;
    g.M = M;
    g.N = N;
    g.K = K;
    g.ldo = ldo;
    g.rope = rope;
    return launch_gemm(g, epilogue, cus, stream) == hipSuccess ? THI_OK : THI_ERR_HIP;
}

// The SwiGLU MLP: gate/up with the SiLU*up epilogue (RMSNorm in front if gamma is given), h in the workspace, the
// down projection (with the residual if given): two launches.  With thi_set_mlp_fusion(1) it is ONE launch where both
// projections would run as row blocks, the down projection's blocks shared between workgroups, and the fused kernel
// is built for the block shapes (the 7B-shaped layer at 17..32 tokens).  Off by default: measured on the 7B shape at
// 32 tokens the single launch takes 58.0 us against 54.3 us for two (70 us while every workgroup executed the
// agent-scope acquire that reading h after the in-kernel rendezvous needs; one workgroup per XCD does now) -- the
// rendezvous and the device-scope stores of h cost more than the kernel boundary they replace.
int run_mlp(const uint16_t* x, const uint16_t* gamma, float eps, const uint16_t* w_gate, const uint16_t* w_up,
            const uint16_t* w_down, const uint16_t* residual, uint16_t* out, int M, int H, int I, const Workspace& ws,
            hipStream_t stream)
{
    const int epi_up = gamma ? EPI_RMSNORM_SWIGLU : EPI_SWIGLU;
    const int cus = device_cu_count();
    if (M <= SKINNY_MAX_M && g_family.load(std::memory_order_relaxed) == 0 && g_mlp_fusion.load(std::memory_order_relaxed)) {
        const int S = pick_rowblock_split(M, H, I, EPI_PLAIN, cus);
        if (S > 1 && mlp_fused_ok(M, H, I, epi_up, cus, S) && pick_decode_kernel(M, I, H, epi_up, cus) == DK_ROWBLOCK &&
            pick_decode_kernel(M, H, I, EPI_PLAIN, cus) == DK_ROWBLOCK) {
            (void)hipGetLastError();
            SkinnyArgs up{}, down{};
            up.x = x; up.gamma = gamma; up.w0 = w_gate; up.w1 = w_up; up.out = ws.h; up.residual = nullptr;
            up.handover = ws.handover; up.counters = ws.counters;
            up.M = M; up.N = I; up.K = H; up.ldo = I; up.tiles = 0; up.kchunks = (H + SK_KC - 1) / SK_KC; up.eps = eps;
            up.rope = RopeArgs{nullptr, nullptr, 0, 2, nullptr};
            up.spin_limit = g_spin_limit.load(std::memory_order_relaxed); up.withhold_flags = 0;
            down = up;
            down.x = ws.h; down.gamma = nullptr; down.w0 = w_down; down.w1 = nullptr; down.out = out; down.residual = residual;
            down.N = H; down.K = I; down.ldo = H; down.kchunks = S; down.eps = 0.f;
            return launch_mlp_fused(up, down, epi_up, cus, stream, S) == hipSuccess ? THI_OK : THI_ERR_HIP;
        }
    }
    int rc = run_projection(x, gamma, eps, w_gate, w_up, ws.h, M, I, H, I, epi_up, ws, stream);
    if (rc != THI_OK) return rc;
    return run_projection(ws.h, nullptr, 0.f, w_down, nullptr, out, M, H, I, H, EPI_PLAIN, ws, stream,
                          RopeArgs{nullptr, nullptr, 0, 2, nullptr}, residual);
}

int check_common(int M, int N, int K, const void* workspace, size_t workspace_bytes, size_t need)
{
    if (M < 1 || N < 1 || K < 1 || (K & 7)) return THI_ERR_SHAPE;
    if (!workspace) return THI_ERR_NULL;
    if (misaligned(workspace, 256)) return THI_ERR_ALIGN;
    if (workspace_bytes < need) return THI_ERR_WORKSPACE;
    return THI_OK;
}

}  // namespace

extern "C" {

int thi_rmsnorm_qkv(const void* x, const void* gamma, float eps, const void* w_qkv, void* out,
                    int M, int N, int K, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!x || !gamma || !w_qkv || !out) return THI_ERR_NULL;
    int rc = check_common(M, N, K, workspace, workspace_bytes, workspace_need(THI_OP_RMSNORM_QKV, M, N, K));
    if (rc != THI_OK) return rc;
    if (misaligned(x, 16) || misaligned(gamma, 16) || misaligned(w_qkv, 16) || misaligned(out, 16)) return THI_ERR_ALIGN;
    Workspace ws = carve(workspace, workspace_bytes, THI_OP_RMSNORM_QKV, M, N, K);
    return run_projection((const uint16_t*)x, (const uint16_t*)gamma, eps, (const uint16_t*)w_qkv, nullptr,
                          (uint16_t*)out, M, N, K, N, EPI_RMSNORM, ws, (hipStream_t)hip_stream);
}

int thi_rmsnorm_qkv_rope(const void* x, const void* gamma, float eps, const void* w_qkv, const int* positions,
                         const float* theta, int n_rot, int head_dim, void* out, int M, int N, int K,
                         void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!x || !gamma || !w_qkv || !out || !positions || !theta) return THI_ERR_NULL;
    int rc = check_common(M, N, K, workspace, workspace_bytes, workspace_need(THI_OP_RMSNORM_QKV, M, N, K));
    if (rc != THI_OK) return rc;
    if (head_dim < 2 || (head_dim & 1) || n_rot < 0 || n_rot > N || (n_rot % head_dim)) return THI_ERR_SHAPE;
    if (misaligned(x, 16) || misaligned(gamma, 16) || misaligned(w_qkv, 16) || misaligned(out, 16) ||
        misaligned(positions, 4) || misaligned(theta, 4))
        return THI_ERR_ALIGN;
    Workspace ws = carve(workspace, workspace_bytes, THI_OP_RMSNORM_QKV, M, N, K);
    return run_projection((const uint16_t*)x, (const uint16_t*)gamma, eps, (const uint16_t*)w_qkv, nullptr,
                          (uint16_t*)out, M, N, K, N, EPI_RMSNORM_ROPE, ws, (hipStream_t)hip_stream,
                          RopeArgs{positions, theta, n_rot, head_dim, nullptr});
}

int thi_linear(const void* x, const void* w, void* out, int M, int N, int K,
               void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!x || !w || !out) return THI_ERR_NULL;
    int rc = check_common(M, N, K, workspace, workspace_bytes, workspace_need(THI_OP_LINEAR, M, N, K));
    if (rc != THI_OK) return rc;
    if (misaligned(x, 16) || misaligned(w, 16) || misaligned(out, 16)) return THI_ERR_ALIGN;
    Workspace ws = carve(workspace, workspace_bytes, THI_OP_LINEAR, M, N, K);
    return run_projection((const uint16_t*)x, nullptr, 0.f, (const uint16_t*)w, nullptr, (uint16_t*)out,
                          M, N, K, N, EPI_PLAIN, ws, (hipStream_t)hip_stream);
}

int thi_swiglu_mlp(const void* x, const void* w_gate, const void* w_up, const void* w_down, void* out,
                   int M, int H, int I, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!x || !w_gate || !w_up || !w_down || !out) return THI_ERR_NULL;
    if (I < 1 || (I & 7)) return THI_ERR_SHAPE;
    int rc = check_common(M, H, H, workspace, workspace_bytes, workspace_need(THI_OP_SWIGLU_MLP, M, H, I));
    if (rc != THI_OK) return rc;
    if (misaligned(x, 16) || misaligned(w_gate, 16) || misaligned(w_up, 16) || misaligned(w_down, 16) ||
        misaligned(out, 16))
        return THI_ERR_ALIGN;
    Workspace ws = carve(workspace, workspace_bytes, THI_OP_SWIGLU_MLP, M, H, I);
    return run_mlp((const uint16_t*)x, nullptr, 0.f, (const uint16_t*)w_gate, (const uint16_t*)w_up, (const uint16_t*)w_down,
                   nullptr, (uint16_t*)out, M, H, I, ws, (hipStream_t)hip_stream);
}

int thi_swiglu_gate_up(const void* x, const void* w_gate, const void* w_up, void* h, int M, int H, int I,
                       void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!x || !w_gate || !w_up || !h) return THI_ERR_NULL;
    if (I < 1 || (I & 7)) return THI_ERR_SHAPE;
    int rc = check_common(M, H, H, workspace, workspace_bytes, workspace_need(THI_OP_SWIGLU_MLP, M, H, I));
    if (rc != THI_OK) return rc;
    if (misaligned(x, 16) || misaligned(w_gate, 16) || misaligned(w_up, 16) || misaligned(h, 16)) return THI_ERR_ALIGN;
    Workspace ws = carve(workspace, workspace_bytes, THI_OP_SWIGLU_MLP, M, H, I);
    return run_projection((const uint16_t*)x, nullptr, 0.f, (const uint16_t*)w_gate, (const uint16_t*)w_up,
                          (uint16_t*)h, M, I, H, I, EPI_SWIGLU, ws, (hipStream_t)hip_stream);
}

int thi_linear_residual(const void* x, const void* w, const void* residual, void* out, int M, int N, int K,
                        void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!x || !w || !residual || !out) return THI_ERR_NULL;
    int rc = check_common(M, N, K, workspace, workspace_bytes, workspace_need(THI_OP_LINEAR, M, N, K));
    if (rc != THI_OK) return rc;
    if (misaligned(x, 16) || misaligned(w, 16) || misaligned(residual, 16) || misaligned(out, 16)) return THI_ERR_ALIGN;
    Workspace ws = carve(workspace, workspace_bytes, THI_OP_LINEAR, M, N, K);
    return run_projection((const uint16_t*)x, nullptr, 0.f, (const uint16_t*)w, nullptr, (uint16_t*)out,
                          M, N, K, N, EPI_PLAIN, ws, (hipStream_t)hip_stream, RopeArgs{nullptr, nullptr, 0, 2, nullptr},
                          (const uint16_t*)residual);
}

int thi_rmsnorm_swiglu_mlp(const void* x, const void* gamma, float eps, const void* w_gate, const void* w_up,
                           const void* w_down, const void* residual, void* out, int M, int H, int I,
                           void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!x || !gamma || !w_gate || !w_up || !w_down || !out) return THI_ERR_NULL;
    if (I < 1 || (I & 7)) return THI_ERR_SHAPE;
    int rc = check_common(M, H, H, workspace, workspace_bytes, workspace_need(THI_OP_SWIGLU_MLP, M, H, I));
    if (rc != THI_OK) return rc;
    if (misaligned(x, 16) || misaligned(gamma, 16) || misaligned(w_gate, 16) || misaligned(w_up, 16) ||
        misaligned(w_down, 16) || misaligned(out, 16) || (residual && misaligned(residual, 16)))
        return THI_ERR_ALIGN;
    Workspace ws = carve(workspace, workspace_bytes, THI_OP_SWIGLU_MLP, M, H, I);
    return run_mlp((const uint16_t*)x, (const uint16_t*)gamma, eps, (const uint16_t*)w_gate, (const uint16_t*)w_up,
                   (const uint16_t*)w_down, (const uint16_t*)residual, (uint16_t*)out, M, H, I, ws, (hipStream_t)hip_stream);
}

size_t thi_attention_workspace_bytes(int B, int Hq, int Hkv, int D, int S_max)
{
    if (B < 1 || Hq < 1 || Hkv < 1 || S_max < 1 || (D != 64 && D != 128) || Hq % Hkv) return 0;
    return fixed_bytes() + round_up((size_t)B * Hq * AT_MAX_SPLIT * (D + 2) * sizeof(float), 256);
}

int thi_decode_attention(const void* q, const void* k_cache, const void* v_cache, const int* seq_lens, float scale,
                         void* out, int B, int Hq, int Hkv, int D, int S_max,
                         void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!q || !k_cache || !v_cache || !seq_lens || !out || !workspace) return THI_ERR_NULL;
    if (B < 1 || Hq < 1 || Hkv < 1 || S_max < 1 || (D != 64 && D != 128) || Hq % Hkv) return THI_ERR_SHAPE;
    if ((long)B * Hkv > 65535L * 8 || B > 65535) return THI_ERR_SHAPE;
    if (misaligned(q, 16) || misaligned(k_cache, 16) || misaligned(v_cache, 16) || misaligned(out, 16) ||
        misaligned(seq_lens, 4) || misaligned(workspace, 256))
        return THI_ERR_ALIGN;
    if (workspace_bytes < thi_attention_workspace_bytes(B, Hq, Hkv, D, S_max)) return THI_ERR_WORKSPACE;
    (void)hipGetLastError();      // an error another user of the runtime left behind is not ours to report
    AttnArgs a{};
    a.q = (const uint16_t*)q;
    a.k = (const uint16_t*)k_cache;
    a.v = (const uint16_t*)v_cache;
    a.seq_lens = seq_lens;
    a.out = (uint16_t*)out;
    // behind the other calls' status words and hand-over slots: a shared workspace keeps them intact
    a.part = reinterpret_cast<float*>(static_cast<char*>(workspace) + fixed_bytes());
    a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.D = D; a.S_max = S_max;
    a.group = Hq / Hkv;
    // cut along the positions only as far as it takes to give every compute unit a workgroup: more,
    // shorter chunks measured slower (32 requests x 8 cache heads x 2048 positions: 52 -> 42 us going from
    // four workgroups per compute unit to one; 8 requests: 28 -> 19 us), and with a workgroup per compute
    // unit already there the second pass is not needed at all
    const int gt = attention_heads_per_workgroup(a.group);
    const int passes = (a.group + gt - 1) / gt;
    const int quantum = attention_chunk_quantum(D, gt);
    const long base = (long)B * Hkv * passes;
    long want = ((long)device_cu_count() + base - 1) / base;
    if (want < 1) want = 1;
    if (want > AT_MAX_SPLIT) want = AT_MAX_SPLIT;
    int chunk = (int)((S_max + want - 1) / want);
    chunk = (chunk + quantum - 1) / quantum * quantum;
    a.chunk = chunk;
    a.nsplit = (S_max + chunk - 1) / chunk;
    a.scale2 = scale * 1.44269504088896340736f;
    return launch_attention(a, (hipStream_t)hip_stream) == hipSuccess ? THI_OK : THI_ERR_HIP;
}

size_t thi_workspace_bytes(int op, int M, int N_or_H, int K_or_I)
{
    if (op < THI_OP_RMSNORM_QKV || op > THI_OP_SWIGLU_MLP) return 0;
    if (M < 1 || N_or_H < 1 || K_or_I < 1) return 0;
    return workspace_need(op, M, N_or_H, K_or_I);
}

int thi_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!workspace) return THI_ERR_NULL;
    if (misaligned(workspace, 256)) return THI_ERR_ALIGN;
    if (workspace_bytes < fixed_bytes()) return THI_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)hip_stream;
    (void)hipGetLastError();      // an error another user of the runtime left behind is not ours to report
    return launch_fill_words(workspace, WS_COUNTER_BYTES, 0u, stream) == hipSuccess ? THI_OK : THI_ERR_HIP;
}

// ---- the entry point that allocates nothing ---------------------------------------------------------
// The decode kernels' scratch memory (status words, then the hand-over slots: the fixed part of a workspace)
// as a file-scope device array.  Each GPU the library runs on holds its own copy until the process ends.
// In host code the array's name is only a stand-in for the symbol: the device address is looked up once
// per device and that pointer is what the kernels are given.
constexpr size_t STATIC_SCRATCH_BYTES = WS_COUNTER_BYTES + (size_t)SK_MAX_GRID * SK_SLOT_WORDS * sizeof(unsigned);
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

int thi_linear_static(const void* x, const void* w, void* out, int M, int N, int K, void* hip_stream)
{
    if (!x || !w || !out) return THI_ERR_NULL;
    if (M < 1 || N < 1 || K < 1 || (K & 7)) return THI_ERR_SHAPE;
    if (M > THI_STATIC_MAX_M) return THI_ERR_SHAPE;       // the static scratch array holds the decode kernels' part only
    if (misaligned(x, 16) || misaligned(w, 16) || misaligned(out, 16)) return THI_ERR_ALIGN;
    if (fixed_bytes() > STATIC_SCRATCH_BYTES) return THI_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)hip_stream;
    (void)hipGetLastError();      // an error another user of the runtime left behind is not ours to report

    // once per device, with that device current: the array's address on this GPU
    static std::mutex lock;
    static void* scratch_ptr[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return THI_ERR_HIP;
    void* ptr;
    {
        std::lock_guard<std::mutex> guard(lock);
        ptr = scratch_ptr[dev];
        if (!ptr) {
            if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return THI_ERR_HIP;
            // the status words must be zero before the first kernel uses them (a fill kernel, so that a
            // caller under stream capture records no memset node); every kernel leaves them zero again
            if (launch_fill_words(ptr, WS_COUNTER_BYTES, 0u, stream) != hipSuccess) return THI_ERR_HIP;
            scratch_ptr[dev] = ptr;
        }
    }
    Workspace ws = carve(ptr, fixed_bytes(), THI_OP_LINEAR, M, N, K);      // decode layout: no GEMM region
    return run_projection((const uint16_t*)x, nullptr, 0.f, (const uint16_t*)w, nullptr, (uint16_t*)out,
                          M, N, K, N, EPI_PLAIN, ws, stream);
}

int thi_workspace_status(const void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!workspace) return THI_ERR_NULL;
    if (misaligned(workspace, 256)) return THI_ERR_ALIGN;
    if (workspace_bytes < fixed_bytes()) return THI_ERR_WORKSPACE;
    (void)hipGetLastError();
    hipStream_t stream = (hipStream_t)hip_stream;
    unsigned marker = 0;
    const unsigned* word = static_cast<const unsigned*>(workspace) + (WS_MAX_COUNTERS - 1);
    if (hipMemcpyAsync(&marker, word, sizeof(marker), hipMemcpyDeviceToHost, stream) != hipSuccess) return THI_ERR_HIP;
    if (hipStreamSynchronize(stream) != hipSuccess) return THI_ERR_HIP;
    return marker ? THI_ERR_TIMEOUT : THI_OK;
}

int thi_debug_handover(unsigned spin_limit, int withhold_flags)
{
    g_spin_limit.store(spin_limit ? spin_limit : SK_SPIN_LIMIT);
    g_withhold_flags.store(withhold_flags ? 1 : 0);
    return THI_OK;
}

const char* thi_status_string(int status)
{
    switch (status) {
    case THI_OK: return "THI_OK";
    case THI_ERR_NULL: return "THI_ERR_NULL: a required pointer is NULL";
    case THI_ERR_SHAPE: return "THI_ERR_SHAPE: extents must be >= 1 and K, H, I multiples of 8";
    case THI_ERR_ALIGN: return "THI_ERR_ALIGN: pointers must be 16-byte aligned (workspace 256-byte)";
    case THI_ERR_WORKSPACE: return "THI_ERR_WORKSPACE: workspace smaller than thi_workspace_bytes()";
    case THI_ERR_HIP: return "THI_ERR_HIP: kernel launch failed";
    case THI_ERR_TIMEOUT: return "THI_ERR_TIMEOUT: a hand-over between workgroups timed out; results undefined, re-initialise the workspace";
    default: return "THI_ERR_UNKNOWN";
    }
}

int thi_version(void) { return THI_VERSION; }

int thi_query_kernel_family(int M, int N, int K, int fused)
{
    if (M < 1 || N < 1 || K < 1 || fused < 0 || fused > 2) return 0;
    const int epilogue = fused == 1 ? EPI_RMSNORM : fused == 2 ? EPI_SWIGLU : EPI_PLAIN;
    const DecodePlan dp = plan_decode(M, N, K, epilogue, device_cu_count());
    return dp.kernel != 0 ? dp.kernel : 2;
}

int thi_set_mlp_fusion(int on) { return g_mlp_fusion.exchange(on ? 1 : 0); }

int thi_set_rowblock_split(int split)
{
    if (split < 0 || split > ROWBLOCK_MAX_SPLIT) split = 0;
    return g_rowblock_split.exchange(split);
}

int thi_set_kernel_family(int family)
{
    if (family < 0 || family > 4) family = 0;
    return g_family.exchange(family);
}

}  // extern "C"
