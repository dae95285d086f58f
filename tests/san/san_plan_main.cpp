// Driver for the host-sanitizer build of the C ABI's pure host part (argument validators, the
// per-call plan, the host id check): walks a grid of valid and invalid arguments; pointers are
// fake addresses that validation must never dereference.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "vt.h"

int main()
{
    void* const fake = reinterpret_cast<void*>(0x1000);
    long long acc = 0;
    const int64_t rows_list[] = {0, 1, 2, 3, 5, 8, 16, 17, 33, 128, 129, 512, 1024, 5000};
    const int64_t H_list[] = {0, 8, 64, 72, 256, 2048, 4096, 8192, 16384, 12};
    const int64_t V_list[] = {0, 1, 5, 100, 4096, 13264, 32000, 128256, 131072, 400000};
    const int k_list[] = {0, 1, 2, 7, 10, 16, 17, 33, 64, 65};
    for (int64_t rows : rows_list)
        for (int64_t H : H_list)
            for (int64_t Vd : V_list)
                for (int k : k_list) {
                    const size_t need = vt_draft_head_workspace_bytes(rows, H, Vd, k);
                    const int regime = vt_draft_head_regime(rows, H, Vd, k);
                    if ((need == 0) != (regime < 0))
                        return 2;
                    const vt_status st = vt_validate_draft_head_args(fake, rows, H, fake, fake, Vd, k, fake, fake, fake, need);
                    if ((st == VT_OK) != (need != 0))
                        return 3;
                    if (need != 0 && vt_validate_draft_head_args(fake, rows, H, fake, fake, Vd, k, fake, fake, fake, need - 1) != VT_ERR_WORKSPACE)
                        return 4;
                    acc += (long long)need + regime;
                }
    for (int64_t V : V_list)
        for (int64_t H : H_list)
            for (int64_t Vd : V_list)
                acc += vt_validate_build_subset_args(fake, V, H, fake, Vd, fake, fake);
    std::vector<int32_t> ids = {5, 1, 999, 0};
    if (vt_check_token_ids_host(ids.data(), (int64_t)ids.size(), 1000) != VT_OK)
        return 5;
    ids.push_back(1000);
    if (vt_check_token_ids_host(ids.data(), (int64_t)ids.size(), 1000) != VT_ERR_ID_RANGE)
        return 6;
    ids.back() = 5;
    if (vt_check_token_ids_host(ids.data(), (int64_t)ids.size(), 1000) != VT_ERR_ID_DUP)
        return 7;
    for (int s = 0; s < 12; ++s)
        acc += vt_status_str((vt_status)s)[0];
    std::printf("san_plan ok checksum=%lld version=%d\n", acc, vt_version());
    return 0;
}
