// Host-side planning arithmetic of libthi: how work is dealt to workgroups and how large the workspace
// regions are.  No kernels and no HIP calls here, so that this file and api.hip can also be built for the
// host alone (with stand-ins for the kernel launchers) and run under the sanitizers on a machine without
// a GPU.
#include "thi_internal.h"

namespace thi {

// ---- decode kernels ------------------------------------------------------------------------------
size_t skinny_handover_bytes() { return (size_t)SK_MAX_GRID * SK_SLOT_WORDS * sizeof(unsigned); }

// Row blocks: the outputs (rows of W, gate/up pairs for SwiGLU) are dealt to the workgroups in equal contiguous
// blocks; a block is T tiles of 16 rows in flight per pass over K (Sec. III-B.2: split the work along N).
RowBlockPlan plan_rowblock(int N, int epilogue, int num_cus, int ksplit)
{
    RowBlockPlan p;
    const int out_per_tile = is_swiglu(epilogue) ? 8 : 16;
    if (ksplit < 1) ksplit = 1;
    int groups = num_cus / ksplit;          // row blocks: ksplit workgroups each
    if (groups < 1) groups = 1;
    int per_wg = (N + groups - 1) / groups;
    if (!is_swiglu(epilogue)) per_wg = (per_wg + 1) & ~1;      // rotary pairs (n, n + 1) stay in one block
    p.per_wg = per_wg;
    p.ksplit = ksplit;
    p.grid = ((N + per_wg - 1) / per_wg) * ksplit;
    p.tiles = (per_wg + out_per_tile - 1) / out_per_tile;
    p.passes = (p.tiles + 5) / 6;
    const int per_pass = (p.tiles + p.passes - 1) / p.passes;
    p.T = per_pass < 2 ? 2 : per_pass;
    return p;
}

bool rowblock_split_ok(int N, int K, int epilogue, int num_cus, int ksplit)
{
    if (ksplit < 2 || ksplit > ROWBLOCK_MAX_SPLIT || epilogue != EPI_PLAIN) return false;
    if (((K + 127) >> 7) < 8 * ksplit) return false;           // every wave of every share gets k of its own
    const RowBlockPlan p = plan_rowblock(N, epilogue, num_cus, ksplit);
    // one pass (the hand-over happens once, at the end), one workgroup per compute unit at most, and a
    // slot / a counter per workgroup / block within the workspace
    return p.passes == 1 && p.grid <= num_cus && p.grid <= SK_MAX_GRID && p.T * 512 <= SK_SLOT_WORDS;
}

// The single-launch decode MLP: which shapes the one fused kernel that is built serves.
bool mlp_fused_ok(int M, int H, int I, int epilogue_up, int num_cus, int ksplit_down)
{
    if (M <= 16 || M > 32 || H < 1024 || H > ROWSLAB_MAX_K || I < 1024 || I > ROWSLAB_MAX_K) return false;
    if (epilogue_up != EPI_SWIGLU && epilogue_up != EPI_RMSNORM_SWIGLU) return false;
    if (epilogue_up == EPI_RMSNORM_SWIGLU && H > 24576) return false;      // gamma in LDS beside the two phases' ~104 KiB
    if (!rowblock_split_ok(H, I, EPI_PLAIN, num_cus, ksplit_down)) return false;
    const RowBlockPlan up = plan_rowblock(I, epilogue_up, num_cus, 1), down = plan_rowblock(H, EPI_PLAIN, num_cus, ksplit_down);
    // the one pair of block shapes that is built: six gate/up tiles and four down tiles in flight, one pass each
    return up.passes == 1 && up.T == 6 && up.grid <= num_cus && down.passes == 1 && down.T == 4 && down.grid <= num_cus &&
           num_cus <= MLP_MAX_GRID;
}

// ---- prefill GEMM ----------------------------------------------------------------------------------
size_t gemm_partial_bytes() { return (size_t)GEMM_MAX_GRID * 2 * 128 * 128 * sizeof(float); }

// ---- decode attention ------------------------------------------------------------------------------
int attention_heads_per_workgroup(int group) { return group >= 8 ? 8 : group >= 4 ? 4 : group >= 2 ? 2 : 1; }

// chunks are whole multiples of this (a multiple of every kernel's positions per workgroup iteration)
int attention_chunk_quantum(int D, int gt)
{
    (void)D; (void)gt;
    return 128;
}

}  // namespace thi
