/*
 * thi.h -- C ABI of libthi: the fp16 linear-operator hot path of a Llama
 * decoder layer on AMD MI355X (gfx950).
 *
 * Numerical contract (paper Sec. III-B.4, "FP16 operator support"): operands
 * are stored as IEEE binary16, products are accumulated in fp32, RMSNorm
 * statistics are kept in fp32, results are rounded to binary16
 * (round-to-nearest-even) once, at the store.
 *
 * Common conventions for every entry point
 *   - Every data pointer is a DEVICE pointer (HIP global memory) to dense,
 *     row-major fp16 data whose innermost extent is contiguous; it must be
 *     16-byte aligned (THI_ERR_ALIGN otherwise).  K (and H, I) must be a
 *     multiple of 8 so that every row starts 16-byte aligned (THI_ERR_SHAPE).
 *     M, N, K >= 1.  Weights are [N,K]: one row per output feature, i.e. the
 *     transpose of the W in the paper's Y = X*W (Sec. III-B.1).
 *   - Ownership: the caller owns every buffer, including `workspace`; the
 *     library allocates nothing, frees nothing and keeps no pointer after the
 *     call returns.  `out` must not overlap any input or the workspace.
 *   - Workspace: at least thi_workspace_bytes(op, ...) bytes, 256-byte
 *     aligned, and prepared ONCE after allocation with thi_workspace_init().
 *     Every call leaves the workspace ready for the next call.  One workspace
 *     must not be used by two calls that may run concurrently.  The decode
 *     kernels (M <= 64) hand partial results from workgroup to workgroup inside
 *     one launch of one workgroup per compute unit, which assumes that all of
 *     them are resident together (true on a GPU the process has to itself); the
 *     waits are bounded, so a launch always terminates, but if the GPU is shared
 *     so heavily (another stream or process, a compute-unit mask) that a wait
 *     runs out, the outputs of that call are undefined and the workspace's
 *     time-out marker is set: thi_workspace_status() reports it as
 *     THI_ERR_TIMEOUT until the workspace is re-initialised.
 *   - Execution: work is enqueued on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = the default stream); the call returns without
 *     synchronising.  Results are bitwise reproducible from run to run.
 *   - Errors: arguments are validated on the host before anything is
 *     launched; a thi_status code is returned (never an exception, abort or
 *     message on stderr).  THI_ERR_HIP reports a failed launch.
 */
#ifndef THI_H
#define THI_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    THI_OK = 0,
    THI_ERR_NULL = 1,      /* a required pointer is NULL */
    THI_ERR_SHAPE = 2,     /* non-positive extent, or K/H/I not a multiple of 8 */
    THI_ERR_ALIGN = 3,     /* a pointer is not 16-byte (workspace: 256-byte) aligned */
    THI_ERR_WORKSPACE = 4, /* workspace smaller than thi_workspace_bytes() */
    THI_ERR_HIP = 5,       /* the HIP runtime refused a launch */
    THI_ERR_TIMEOUT = 6    /* thi_workspace_status: a hand-over between workgroups ran out of time */
} thi_status;

typedef enum {
    THI_OP_RMSNORM_QKV = 0,
    THI_OP_LINEAR = 1,
    THI_OP_SWIGLU_MLP = 2
} thi_op;

/*
 * RMSNorm fused in front of the QKV projection: the "[low-density] -
 * high-density" half of the paper's fusion unit (Sec. III-C.1), with the
 * statistics in fp32 (Sec. III-B.4).
 *
 *   r[m]     = 1 / sqrt( (1/K) * sum_k x[m,k]^2 + eps )
 *   out[m,n] = sum_k ( x[m,k] * r[m] * gamma[k] ) * w_qkv[n,k]
 *
 * x [M,K], gamma [K], w_qkv [N,K] (rows of Wq, Wk, Wv stacked; grouped-query
 * attention only changes N), out [M,N]; all fp16 device memory.  Up to 64
 * tokens the normalised activations are never written to memory (the decode
 * kernels scale x by gamma on its way to the matrix cores and apply r[m] to the
 * accumulator); where the GEMM kernels run (M > 64, some shapes from 33) a
 * small pass of its own writes them to the workspace once, as fp16.
 */
int thi_rmsnorm_qkv(const void* x, const void* gamma, float eps, const void* w_qkv,
                    void* out, int M, int N, int K,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * thi_rmsnorm_qkv with the rotary position embedding fused behind it (the paper's worked example
 * of the fusion rule, Algorithm 1 "Linear-RoPE fusion": the rotation is applied to the accumulator
 * before the store).  Columns [0, n_rot) of the output -- the Q and K projections -- are rotated in
 * interleaved pairs (2i, 2i+1) within each head of head_dim columns:
 *
 *   ang = positions[m] * theta[i],  i = (n mod head_dim) / 2
 *   out[m,2i'] = y[2i'] cos(ang) - y[2i'+1] sin(ang),  out[m,2i'+1] = y[2i'+1] cos(ang) + y[2i'] sin(ang)
 *
 * with y the thi_rmsnorm_qkv result in fp32.  positions [M] int32 and theta [head_dim/2] fp32 are
 * device memory (4-byte aligned); n_rot must be a multiple of head_dim (even) and <= N; columns
 * >= n_rot (V) are not rotated.  Everything else as thi_rmsnorm_qkv.  Above 32 tokens the cosines and
 * sines come from a table in the workspace that the call fills first, which holds head_dim <= 256
 * (THI_ERR_SHAPE beyond); the decode kernels take any head_dim.
 */
int thi_rmsnorm_qkv_rope(const void* x, const void* gamma, float eps, const void* w_qkv,
                         const int* positions, const float* theta, int n_rot, int head_dim,
                         void* out, int M, int N, int K,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The linear operator (Sec. III-B.1; decode shapes follow the small-M rule of
 * Sec. III-B.2: broadcast X, split N):  out[m,n] = sum_k x[m,k] * w[n,k].
 * x [M,K], w [N,K], out [M,N]; all fp16 device memory.
 */
int thi_linear(const void* x, const void* w, void* out, int M, int N, int K,
               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * thi_linear for callers that cannot allocate or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same operator and same kernels as
 * thi_linear for up to THI_STATIC_MAX_M tokens (the weight-streaming decode kernels), bit-identical
 * results; the kernels' scratch memory (status words and hand-over slots, about 17 MiB) is a static
 * device array inside the library instead of a caller's workspace.  The call allocates and frees
 * nothing.  M > THI_STATIC_MAX_M returns THI_ERR_SHAPE (the GEMM kernels' scratch is not held
 * statically); with thi_set_kernel_family(2) in force every call returns THI_ERR_WORKSPACE.
 * Every GPU the library is used on holds its own copy of the array until the process ends.  All
 * calls on one GPU share that array: calls that may overlap on one GPU (different streams) race;
 * calls on one stream, or otherwise ordered, are fine.  The first call on a device also enqueues a
 * small clearing kernel in front of the operator, on `hip_stream`.
 */
#define THI_STATIC_MAX_M 32
int thi_linear_static(const void* x, const void* w, void* out, int M, int N, int K, void* hip_stream);

/*
 * SwiGLU MLP with SiLU(gate)*up fused behind the gate/up projections (the
 * "high-density - [low-density]" half of the fusion unit, Sec. III-C.1):
 *
 *   g[m,j]   = sum_k x[m,k] * w_gate[j,k],   u[m,j] = sum_k x[m,k] * w_up[j,k]
 *   h[m,j]   = g / (1 + exp(-g)) * u          (fp32; stored once as fp16 in the workspace)
 *   out[m,n] = sum_j h[m,j] * w_down[n,j]
 *
 * x [M,H], w_gate and w_up [I,H], w_down [H,I], out [M,H]; all fp16 device
 * memory.  g and u are never written to HBM.
 *
 * Placement hint (performance only, any placement is correct): the decode
 * kernel streams the same rows of w_gate and w_up at the same time.  With
 * w_up a whole multiple of 2 MiB behind w_gate -- what an allocator that
 * hands out large buffers on 2 MiB boundaries produces -- it measured 1-2 %
 * slower than with w_up some tens of KiB off such a multiple (7B shape at 32
 * tokens: 31.3 against 31.0 us; bench.py places w_up 64 KiB past the end of
 * w_gate).
 */
int thi_swiglu_mlp(const void* x, const void* w_gate, const void* w_up, const void* w_down,
                   void* out, int M, int H, int I,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * First half of thi_swiglu_mlp on its own: h[m,j] = silu(x w_gate^T) * (x w_up^T),
 * h [M,I] fp16 device memory owned by the caller (Sec. III-C.1, linear operator
 * followed by a low-density one).  Useful when the down projection is sharded
 * differently, and to time the layer's largest kernel in isolation.  Workspace:
 * as for thi_swiglu_mlp with the same (M, H, I).
 */
int thi_swiglu_gate_up(const void* x, const void* w_gate, const void* w_up, void* h,
                       int M, int H, int I,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The two operators that close the residual blocks of the decoder layer
 * (Sec. III-D.3: norm -> attention -> norm -> FFN; Sec. III-C.1: a low-density
 * operator behind the linear one is applied to the accumulator before the store).
 *
 * thi_linear_residual:   out[M,N] = residual[M,N] + x[M,K] * w[N,K]^T
 *     the O projection and any projection that ends a residual block; the sum
 *     is formed in fp32 and rounded once.
 * thi_rmsnorm_swiglu_mlp: out[M,H] = residual[M,H] + (silu(n Wg^T) * (n Wu^T)) Wd^T
 *     with n = rmsnorm(x; gamma, eps) never materialised (the post-attention
 *     normalisation fused in front of the gate/up projections, as RMSNorm is in
 *     thi_rmsnorm_qkv).  residual may be NULL (nothing is added).
 * `residual` is fp16 [M,N] resp. [M,H], 16-byte aligned; it MAY be the same
 * buffer as `out` (every element is read before it is written, by the same
 * thread), but must not otherwise overlap it.  Workspace: as for thi_linear
 * resp. thi_swiglu_mlp.  Everything else as in the common conventions.
 */
int thi_linear_residual(const void* x, const void* w, const void* residual, void* out,
                        int M, int N, int K,
                        void* workspace, size_t workspace_bytes, void* hip_stream);
int thi_rmsnorm_swiglu_mlp(const void* x, const void* gamma, float eps, const void* w_gate, const void* w_up,
                           const void* w_down, const void* residual, void* out,
                           int M, int H, int I,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Decode attention for a batch of requests that each add one token to their own
 * key/value cache (Eq. 6: softmax(Q K^T / sqrt(d)) V per head; Sec. III-D.1: the
 * attention part of a batch is run request by request because the caches differ;
 * Sec. III-C.2: Q and O stay on chip, K and V stream by once).
 *
 *   out[b,h,:] = sum_j p_j * v[b,g,j,:],  p = softmax_j(scale * q[b,h,:] . k[b,g,j,:]),
 *   j over [0, seq_lens[b]),  g = h / (Hq/Hkv)   (grouped-query attention; Hkv = Hq is plain
 *   multi-head attention)
 *
 * q [B,Hq,D], out [B,Hq,D], k_cache and v_cache [B,Hkv,S_max,D] (the positions of one head
 * are contiguous), all fp16 device memory, 16-byte aligned; seq_lens [B] int32 DEVICE memory,
 * 0 <= seq_lens[b] <= S_max (not checked on the host; a request with 0 positions gets a zero
 * row; cache contents at positions >= seq_lens[b] are never used).  The cache must already hold
 * the current token's key and value.  D is 64 or 128, Hq a multiple of Hkv (THI_ERR_SHAPE
 * otherwise).  scale is usually 1/sqrt(D).  Scores, weights and sums are fp32; one fp16 rounding
 * at the end.  Workspace: thi_attention_workspace_bytes(), 256-byte aligned, no preparation
 * needed; it may be the (prepared) workspace of the other calls if large enough: the partial results
 * lie behind the status words and hand-over slots of those calls, which are left untouched.
 * Reproducible bit for bit.
 */
size_t thi_attention_workspace_bytes(int B, int Hq, int Hkv, int D, int S_max);
int thi_decode_attention(const void* q, const void* k_cache, const void* v_cache, const int* seq_lens, float scale,
                         void* out, int B, int Hq, int Hkv, int D, int S_max,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Bytes of workspace the given operator needs for the given shape
 * (op = thi_op; (M, N, K) for the first two operators, (M, H, I) for the MLP).
 * Pure host arithmetic: touches no device.  Returns 0 for invalid arguments.
 * Up to 32 tokens (the decode kernels) this is the fixed part -- 64 KiB of status
 * words and about 17 MiB of hand-over slots -- plus M*I*2 bytes for the MLP;
 * above, 256 MiB for the GEMM kernels' partial tiles and the buffers of the
 * prefill path are added (also below 33 tokens while thi_set_kernel_family(2) is
 * in force).  A call whose kernel needs the larger layout on a workspace that
 * lacks it returns THI_ERR_WORKSPACE.
 */
size_t thi_workspace_bytes(int op, int M, int N_or_H, int K_or_I);

/*
 * Prepare a freshly allocated workspace (device pointer, 256-byte aligned):
 * enqueues a small fill kernel on `hip_stream` that zeroes the status words
 * (hand-over flags, arrival counters) the split-K reductions use.
 * `workspace_bytes` must be what thi_workspace_bytes() returned (at least its
 * fixed part, about 17 MiB; THI_ERR_WORKSPACE otherwise).  Needed once per
 * allocation (and again only if a call on that workspace was aborted half-way).
 */
int thi_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Has a hand-over between workgroups timed out on this workspace since it was
 * last initialised (see the workspace conventions above)?  Copies the marker
 * word to the host behind everything enqueued on `hip_stream` and WAITS for that
 * stream.  Returns THI_OK, THI_ERR_TIMEOUT (the outputs of some earlier call on
 * this workspace are undefined; re-initialise it), or an argument / HIP error.
 */
int thi_workspace_status(const void* workspace, size_t workspace_bytes, void* hip_stream);

/* Human-readable name of a thi_status value (static storage). */
const char* thi_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int thi_version(void);

/*
 * The three thi_set_* / thi_debug_* switches below are PROCESS-GLOBAL
 * diagnostics (atomics read by every later call of any thread); they are not
 * needed for normal use and are not meant to be toggled while calls are in
 * flight on other threads.
 *
 * Tuning/diagnostic hook used by the benchmark and tests: force a kernel
 * family for subsequent calls from this process.  family: 0 = automatic
 * (default: a decode kernel up to 32 tokens, the stream-K decode kernel or the
 * GEMM kernels for 33..64 tokens, the GEMM kernels above), 1 = weight-streaming
 * decode kernel with stream-K units (up to 64 tokens per launch),
 * 2 = MFMA GEMM kernels, 3 = weight-streaming decode kernel with row slabs
 * (16 rows over the whole of K per workgroup at a time), 4 = weight-streaming
 * decode kernel with row blocks (N / #CUs rows per workgroup, several 16-row
 * tiles in flight); 3 and 4 fall back to 1 where K < 1024 or K > 32768.
 * Returns the previous setting.  Not needed for normal use.
 */
int thi_set_kernel_family(int family);

/*
 * Tuning/diagnostic hook like the one above, for the row-block decode kernel: the
 * number of workgroups that share one block of rows, each taking 1/split of the
 * reduction dimension (their sums meet through the workspace).  split: 0 = chosen
 * by the library per call (default), 1 = never share, 2..6 = share wherever the
 * shape admits it (plain linear operator, K >= 1024 * split, at most 6 tiles of
 * 16 rows per block), else as 1.  Returns the previous setting.
 */
int thi_set_rowblock_split(int split);

/*
 * Opt-in: on != 0 lets thi_swiglu_mlp / thi_rmsnorm_swiglu_mlp run as ONE launch -- gate/up, a grid-wide rendezvous
 * on h inside the kernel, the down projection (the paper's unified kernel scheduling, Sec. III-C.4) -- where the
 * library has that kernel for the shape (the 7B-shaped layer at 17..32 tokens); 0 (default) = always two launches,
 * which measured faster on MI355X.  Results are identical bit for bit either way.  The single launch keeps its
 * rendezvous tags in status words 2047..2575 of the workspace, which are then not zero between calls (every other
 * status word is); like the other in-kernel hand-overs it needs all workgroups resident at once and reports a
 * time-out through thi_workspace_status().  Returns the previous setting.
 */
int thi_set_mlp_fusion(int on);

/*
 * Test hook for the time-out path of the stream-K decode kernel's hand-over:
 * spin_limit = polls of a contributor's flag before the finishing workgroup
 * gives up (0 = the default, 2^24); withhold_flags != 0 makes the contributors
 * keep their flags down, so that the give-up is certain and every kernel still
 * exits normally.  Returns THI_OK.
 */
int thi_debug_handover(unsigned spin_limit, int withhold_flags);

/*
 * Diagnostic: the kernel family (numbered as above, never 0 for valid arguments)
 * that a call with these extents would run under the current setting.
 * fused: 0 = plain linear operator, 1 = RMSNorm in front, 2 = gate/up with the
 * SwiGLU epilogue (N = I rows per matrix).  Returns 0 for invalid arguments.
 * Reads the current device's compute-unit count; launches nothing.
 */
int thi_query_kernel_family(int M, int N, int K, int fused);

#ifdef __cplusplus
}
#endif
#endif /* THI_H */
