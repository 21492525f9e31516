// Sanitizer driver for the host side of libthi (test infrastructure): api.hip + plan.hip linked against the
// stand-in launchers of api_stubs.cpp.  Sweeps the entry points over invalid arguments (status codes, no
// launch) and over a grid of valid shapes with fake device pointers (never dereferenced: nothing is
// launched), so that every branch of the validation, the workspace layout and the kernel-choice arithmetic
// runs under AddressSanitizer / UndefinedBehaviorSanitizer.  Prints "ok <calls>" on a clean run.
#include "../../include/thi.h"

#include <cstdint>
#include <cstdio>
#include <cstdlib>

namespace thi { int stub_launch_count(); }

#define EXPECT(cond)                                                         \
    do {                                                                     \
        if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } \
    } while (0)

int main()
{
    // fake, suitably aligned "device" addresses: validation looks at alignment only
    void* p = reinterpret_cast<void*>(uintptr_t(0x7f0000000000ull));
    void* q = reinterpret_cast<void*>(uintptr_t(0x7f1000000000ull));
    void* odd = reinterpret_cast<void*>(uintptr_t(0x7f0000000002ull));
    const size_t big = size_t(1) << 40;
    long calls = 0;

    EXPECT(thi_version() >= 100);
    for (int s = -1; s < 9; ++s) EXPECT(thi_status_string(s) != nullptr);
    EXPECT(thi_linear(nullptr, p, p, 1, 8, 8, p, big, nullptr) == THI_ERR_NULL);
    EXPECT(thi_linear(p, p, p, 0, 8, 8, p, big, nullptr) == THI_ERR_SHAPE);
    EXPECT(thi_linear(p, p, p, 1, 8, 12, p, big, nullptr) == THI_ERR_SHAPE);
    EXPECT(thi_linear(odd, p, p, 1, 8, 8, p, big, nullptr) == THI_ERR_ALIGN);
    EXPECT(thi_linear(p, p, p, 1, 8, 8, p, 1024, nullptr) == THI_ERR_WORKSPACE);
    EXPECT(thi_workspace_init(nullptr, big, nullptr) == THI_ERR_NULL);
    EXPECT(thi_workspace_init(p, 16, nullptr) == THI_ERR_WORKSPACE);
    EXPECT(thi_workspace_init(p, big, nullptr) == THI_OK);
    EXPECT(thi_workspace_bytes(7, 1, 8, 8) == 0 && thi_workspace_bytes(0, 0, 8, 8) == 0);
    EXPECT(thi_attention_workspace_bytes(2, 8, 3, 128, 100) == 0);
    EXPECT(thi_rmsnorm_qkv_rope(p, p, 1e-6f, p, (const int*)p, (const float*)p, 24, 16, p, 4, 64, 64, p, big, nullptr) == THI_ERR_SHAPE);
    EXPECT(thi_linear_static(p, p, p, 33, 64, 64, nullptr) == THI_ERR_SHAPE);
    EXPECT(thi_query_kernel_family(0, 8, 8, 0) == 0);

    const int Ms[] = {1, 2, 4, 5, 8, 16, 17, 31, 32, 33, 48, 49, 64, 65, 100, 128, 129, 200, 256, 257, 512, 1000, 1024, 2048, 4096};
    const int Ns[] = {8, 16, 100, 512, 1000, 1536, 4096, 5120, 8192, 10240, 12288, 32000, 152064};
    const int Ks[] = {8, 64, 520, 1024, 1376, 4096, 6656, 8192, 11008, 24576, 28672, 32768, 65536};
    for (int family = 0; family <= 4; ++family) {
        thi_set_kernel_family(family);
        for (int split = 0; split <= 6; split += (family == 4 || family == 0) ? 1 : 7) {
            thi_set_rowblock_split(split);
            for (int M : Ms)
                for (int N : Ns)
                    for (int K : Ks) {
                        const size_t need = thi_workspace_bytes(THI_OP_LINEAR, M, N, K);
                        EXPECT(need >= (size_t(16) << 20));
                        int rc = thi_linear(p, q, p, M, N, K, p, need, nullptr);
                        EXPECT(rc == THI_OK || rc == THI_ERR_SHAPE);
                        EXPECT(thi_linear(p, q, p, M, N, K, p, need - 1, nullptr) == THI_ERR_WORKSPACE);
                        rc = thi_linear_residual(p, q, q, p, M, N, K, p, need, nullptr);
                        EXPECT(rc == THI_OK || rc == THI_ERR_SHAPE);
                        const size_t need_q = thi_workspace_bytes(THI_OP_RMSNORM_QKV, M, N, K);
                        rc = thi_rmsnorm_qkv(p, q, 1e-6f, q, p, M, N, K, p, need_q, nullptr);
                        EXPECT(rc == THI_OK || rc == THI_ERR_SHAPE);
                        if (N % 64 == 0) {
                            rc = thi_rmsnorm_qkv_rope(p, q, 1e-6f, q, (const int*)q, (const float*)q, N / 64 * 64, 64, p, M, N, K,
                                                      p, need_q, nullptr);
                            EXPECT(rc == THI_OK || rc == THI_ERR_SHAPE);
                        }
                        EXPECT(thi_query_kernel_family(M, N, K, 0) >= 1 && thi_query_kernel_family(M, N, K, 2) >= 1);
                        if (N <= 32768 && K <= 32768) {      // (H, I) of an MLP
                            const size_t need_m = thi_workspace_bytes(THI_OP_SWIGLU_MLP, M, K, N);
                            EXPECT(need_m >= need_q - need_q + (size_t)M * N * 2);
                            rc = thi_swiglu_mlp(p, q, q, q, p, M, K, N, p, need_m, nullptr);
                            EXPECT(rc == THI_OK || rc == THI_ERR_SHAPE);
                            rc = thi_swiglu_gate_up(p, q, q, p, M, K, N, p, need_m, nullptr);
                            EXPECT(rc == THI_OK || rc == THI_ERR_SHAPE);
                            rc = thi_rmsnorm_swiglu_mlp(p, q, 1e-6f, q, q, q, (M & 1) ? q : nullptr, p, M, K, N, p, need_m, nullptr);
                            EXPECT(rc == THI_OK || rc == THI_ERR_SHAPE);
                        }
                        calls += 8;
                    }
        }
    }
    thi_set_kernel_family(0);
    thi_set_rowblock_split(0);
    // decode attention: the chunking arithmetic over request counts, head groupings and context lengths
    for (int B : {1, 2, 7, 8, 32, 64, 1000})
        for (int Hkv : {1, 8, 32})
            for (int g : {1, 2, 4, 5, 8})
                for (int D : {64, 128})
                    for (int S : {1, 100, 2048, 8192, 131072}) {
                        const size_t need = thi_attention_workspace_bytes(B, Hkv * g, Hkv, D, S);
                        EXPECT(need > 0);
                        EXPECT(thi_decode_attention(p, q, q, (const int*)q, 0.1f, p, B, Hkv * g, Hkv, D, S, p, need, nullptr) == THI_OK);
                        EXPECT(thi_decode_attention(p, q, q, (const int*)q, 0.1f, p, B, Hkv * g, Hkv, D, S, p, need - 1, nullptr) == THI_ERR_WORKSPACE);
                        ++calls;
                    }
    EXPECT(thi::stub_launch_count() > 0);
    std::printf("ok %ld\n", calls);
    return 0;
}
