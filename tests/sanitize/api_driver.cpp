// Driver for the host-sanitizer build of the C-ABI library (tests/test_sanitizers.py): everything
// the library does on the host BEFORE its first HIP call -- geometry, workspace carving, plan
// strings, option handling, argument validation -- under AddressSanitizer and UBSan.  No kernel
// is launched and no GPU is needed: every compute call below is one that must be refused.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "flashkm.h"

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "CHECK failed line %d: %s (%s)\n", __LINE__, #c, fk_last_error()); return 1; } } while (0)

int main() {
    const fk_dtype types[3] = {FK_F32, FK_F16, FK_BF16};
    const int Bs[] = {1, 2, 32, 300, 65535, 65536, 0};
    const int64_t Ns[] = {1, 31, 4096, 4097, 100000, (int64_t)1 << 20, ((int64_t)1 << 24) + 5, (int64_t)1 << 28, (int64_t)1 << 31, 0};
    const int ds[] = {1, 3, 8, 12, 64, 100, 128, 136, 256, 512, 513, 0};
    const int Ks[] = {1, 16, 32, 33, 256, 257, 2048, 2049, 65536, 65537, 0};
    char buf[1024], tiny[8];
    size_t shapes = 0;
    for (fk_dtype t : types)
        for (int B : Bs)
            for (int64_t N : Ns)
                for (int d : ds)
                    for (int K : Ks) {
                        const size_t w = fk_workspace_bytes(B, N, d, K, t);
                        const int rc = fk_plan(B, N, d, K, t, buf, sizeof(buf));
                        CHECK((w == 0) == (rc != FK_OK));
                        CHECK(strlen(buf) < sizeof(buf));
                        CHECK(w % 256 == 0);
                        (void)fk_plan(B, N, d, K, t, tiny, sizeof(tiny));    // truncation must stay in bounds
                        CHECK(strlen(tiny) < sizeof(tiny));
                        if (N > 0 && N <= ((int64_t)1 << 24)) (void)fk_ooc_workspace_bytes(N, d, K, t);
                        ++shapes;
                    }
    CHECK(fk_plan(1, 100, 8, 4, FK_F16, nullptr, 0) == FK_EINVAL);
    // options: unknown names, out-of-range values, and each known one there and back
    CHECK(fk_set_option(nullptr, 0) == FK_EINVAL);
    CHECK(fk_set_option("no_such_option", 1) == FK_EINVAL);
    CHECK(fk_set_option("assign_variant", 17) == FK_EINVAL);
    const char* names[] = {"assign_variant", "assign_stream", "sort_stage_bins", "sort_min_rounds", "fused_update", "timer_repeat"};
    for (const char* n : names) {
        CHECK(fk_set_option(n, 1) == FK_OK);
        (void)fk_workspace_bytes(1, 100000, 64, 100, FK_F16);
        (void)fk_plan(1, 100000, 64, 100, FK_F16, buf, sizeof(buf));
        CHECK(fk_set_option(n, -1) == FK_OK);
    }
    // argument validation: all of these must be refused before anything is dereferenced or launched
    alignas(256) static char mem[1 << 16];
    void* p = mem;
    void* odd = mem + 4;
    CHECK(fk_assign(nullptr, p, (int32_t*)p, nullptr, 1, 16, 16, 2, FK_F16, p, sizeof(mem), nullptr) == FK_EINVAL);
    CHECK(fk_assign(p, odd, (int32_t*)p, nullptr, 1, 16, 16, 2, FK_F16, p, sizeof(mem), nullptr) == FK_EINVAL);
    CHECK(fk_assign(p, p, (int32_t*)p, nullptr, 1, 16, 16, 2, FK_F16, odd, sizeof(mem), nullptr) == FK_EINVAL);
    CHECK(fk_assign(p, p, (int32_t*)p, nullptr, 1, 16, 600, 2, FK_F16, p, sizeof(mem), nullptr) == FK_EUNSUPPORTED);
    CHECK(fk_assign(p, p, (int32_t*)p, nullptr, 1, 1 << 20, 128, 1024, FK_F16, p, 1024, nullptr) == FK_EWORKSPACE);
    CHECK(fk_assign(p, p, (int32_t*)p, nullptr, 1, 16, 16, 2, (fk_dtype)9, p, sizeof(mem), nullptr) == FK_EINVAL);
    CHECK(fk_update(p, (int32_t*)p, (float*)p, (float*)p, nullptr, nullptr, 1, 16, 16, 2, FK_F16, p, sizeof(mem), nullptr) == FK_EINVAL);
    CHECK(fk_lloyd_iter(p, (float*)p, nullptr, (int32_t*)p, (int32_t*)p, 1, 16, 16, 2, FK_F16, -1, p, sizeof(mem), nullptr) == FK_EINVAL);
    CHECK(fk_lloyd_iter(p, (float*)p, nullptr, (int32_t*)p, (int32_t*)p, 1, 16, 16, 2, FK_F16, 0, p, sizeof(mem), nullptr) == FK_OK);
    CHECK(fk_sort_inverse((int32_t*)p, (int32_t*)p, (int32_t*)p, 1, 100, 70000, p, sizeof(mem), nullptr) == FK_EUNSUPPORTED);
    CHECK(fk_sort_inverse((int32_t*)p, (int32_t*)p, (int32_t*)p, 1, 100000, 70, p, 64, nullptr) == FK_EWORKSPACE);
    CHECK(fk_lloyd_ooc(nullptr, (float*)p, nullptr, (int32_t*)p, 100, 16, 4, FK_F16, 1, 0, p, sizeof(mem), nullptr) == FK_EINVAL);
    CHECK(fk_lloyd_ooc(p, (float*)p, nullptr, (int32_t*)p, 100, 16, 4, FK_F16, 1, 0, p, sizeof(mem), nullptr) == FK_EINVAL);   // not pinned
    CHECK(fk_standard_assign(p, p, nullptr, (int32_t*)p, 1, 16, 16, 2, FK_F16, p, sizeof(mem), nullptr) == FK_EINVAL);
    CHECK(fk_standard_update(p, (int32_t*)p, (float*)p, (float*)p, (int32_t*)p, nullptr, 1, 16, 16, 2, FK_F16, nullptr) == FK_EINVAL);
    CHECK(fk_assign_static(p, p, (int32_t*)p, nullptr, 1, 1000, 256, 65536, FK_F16, nullptr) == FK_EWORKSPACE);
    CHECK(fk_assign_static(p, p, (int32_t*)p, nullptr, 1, 1000, 12, 16, FK_F16, nullptr) == FK_EUNSUPPORTED);
    CHECK(fk_assign_static(nullptr, p, (int32_t*)p, nullptr, 1, 1000, 16, 16, FK_F16, nullptr) == FK_EINVAL);
    CHECK(fk_assign_static_limit() == ((size_t)16 << 20));
    double ms[4];
    int launches[4];
    fk_stage_timer_start();
    CHECK(fk_stage_timer_stop(ms, launches) == 0);
    CHECK(strlen(fk_last_error()) < 512);
    printf("api sanitizer run ok (%zu shapes)\n", shapes);
    return 0;
}
