// Drives the argument validation of every entry point of the C ABI with fake device pointers (never dereferenced:
// validation fails before any HIP call); built, together with the library's host code, with
// -fsanitize=address,undefined by tests/test_sanitizers_cpu.py.
#include "../../include/slimspec.h"
#include <cstdio>

int main()
{
    void *fake = reinterpret_cast<void *>(0x1000);
    int32_t *fi = reinterpret_cast<int32_t *>(0x1000);
    float *ff = reinterpret_cast<float *>(0x1000);
    slimspec_shape good{600, 4096, 512, 128256}, bad{600, 4100, 512, 128256};
    int32_t off[4] = {0, 100, 100, 600}, off_bad[4] = {0, 200, 100, 600};
    long acc = 0;
    for (int k : {0, 1, 10, 16, 17, 64, 65}) {
        acc += (long)slimspec_workspace_bytes(&good, k) + (long)slimspec_workspace_bytes(&bad, k) + (long)routed_workspace_bytes(&good, k);
        acc += slimspec_head_topk(fake, fake, fake, &good, k, fi, ff, fake, 1024, nullptr);
        acc += slimspec_head_topk(fake, nullptr, fake, &good, k, fi, ff, fake, (size_t)1 << 40, nullptr);
        acc += full_head_topk(fake, fake, SLIMSPEC_BF16, &bad, k, fi, ff, fake, (size_t)1 << 40, nullptr);
        acc += full_head_topk(fake, fake, SLIMSPEC_F32, &good, k, fi, ff, fake, 1024, nullptr);
        acc += truncated_head_topk(fake, fake, SLIMSPEC_BF16, nullptr, &good, k, fi, ff, fake, 1024, nullptr);
        acc += truncated_head_topk(fake, fake, SLIMSPEC_BF16, fi, &good, k, fi, ff, fake, 1024, nullptr);
        acc += slimspec_head_topk_positions(fake, fake, 3, off, fake, &good, k, fi, ff, fake, 1024, nullptr);
        acc += slimspec_head_topk_positions(fake, fake, 3, off_bad, fake, &good, k, fi, ff, fake, 1024, nullptr);
        acc += slimspec_head_sample(fake, fake, fake, &good, k, 5, fi, ff, nullptr, fi, ff, fake, (size_t)1 << 40, nullptr);
        acc += slimspec_head_sample(fake, fake, fake, &good, k, 5, fi, ff, ff, fi, ff, fake, 1024, nullptr);
        acc += full_head_sample(fake, fake, SLIMSPEC_BF16, &good, k, 5, fi, ff, ff, fi, ff, fake, 1024, nullptr);
        acc += routed_head_topk(fake, fake, fake, fake, SLIMSPEC_BF16, &good, k, k, fi, ff, fake, 1024, nullptr);
        acc += slimspec_head_topk_static(fake, fake, nullptr, &good, k, fi, ff, nullptr);
    }
    slimspec_shape huge{4096, 8192, 2048, 8192};
    acc += slimspec_head_topk_static(fake, fake, fake, &huge, 10, fi, ff, nullptr);
    for (int s = -6; s <= 0; ++s) acc += slimspec_status_string(s)[0];
    acc += slimspec_last_hip_error()[0] + slimspec_set_timing_events(fake, nullptr) + slimspec_version();
    std::printf("checksum %ld\n", acc);
    return 0;
}
