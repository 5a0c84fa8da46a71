// Drives the host-only part of the C ABI (slicing, argument validation) under AddressSanitizer +
// UndefinedBehaviorSanitizer on the CPU: every call here returns before the library touches a GPU.
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "mlpmoe.h"

int main()
{
    int bad = 0;
    // slicing: many (d_inter, B, K, pad) combinations with and without a keep list, exact capacity
    for (int d_inter : {0, 5, 100, 4864, 14336})
        for (int B : {1, 3, 8, 16, 64})
            for (int K : {0, 1, B / 2, B})
                for (int pad : {1, 8, 64}) {
                    std::vector<int32_t> off(B + 1);
                    std::vector<float> alpha(B);
                    std::vector<uint8_t> mask(B), keep(d_inter ? d_inter : 1);
                    for (int j = 0; j < d_inter; ++j) keep[j] = (uint8_t)((j * 2654435761u >> 7) % 4 != 0);
                    const int cap = d_inter + B * (pad - 1);
                    std::vector<int32_t> gather(cap ? cap : 1);
                    for (int with_keep = 0; with_keep < 2; ++with_keep) {
                        int rc = mlpmoe_slice(d_inter, B, K, with_keep ? keep.data() : nullptr, pad, off.data(), alpha.data(),
                                              mask.data(), gather.data(), cap);
                        if (rc != MLPMOE_OK || off[0] != 0 || off[B] > cap) ++bad;
                        for (int b = 0; b < B; ++b)
                            if ((off[b + 1] - off[b]) % pad) ++bad;
                        // one entry too few must be refused, not overrun
                        if (off[B] > 0 &&
                            mlpmoe_slice(d_inter, B, K, with_keep ? keep.data() : nullptr, pad, off.data(), alpha.data(),
                                         mask.data(), gather.data(), off[B] - 1) != MLPMOE_ERR_SHAPE)
                            ++bad;
                        // the row count rounded up as well: exact capacity accepted, one entry less refused
                        const int rows_to = 64, cap_r = cap + rows_to - 1;
                        std::vector<int32_t> gather_r(cap_r);
                        rc = mlpmoe_slice_rows(d_inter, B, K, with_keep ? keep.data() : nullptr, pad, rows_to, off.data(),
                                               alpha.data(), mask.data(), gather_r.data(), cap_r);
                        if (rc != MLPMOE_OK || off[B] % rows_to || off[B] > cap_r) ++bad;
                        const int need = off[B];
                        if (need > 0) {
                            std::vector<int32_t> exact(need);
                            if (mlpmoe_slice_rows(d_inter, B, K, with_keep ? keep.data() : nullptr, pad, rows_to, off.data(),
                                                  alpha.data(), mask.data(), exact.data(), need) != MLPMOE_OK)
                                ++bad;
                            if (mlpmoe_slice_rows(d_inter, B, K, with_keep ? keep.data() : nullptr, pad, rows_to, off.data(),
                                                  alpha.data(), mask.data(), exact.data(), need - 1) != MLPMOE_ERR_SHAPE)
                                ++bad;
                        }
                    }
                }
    // validation of the forward entry points: errors are reported before any device access
    int32_t off[3] = {0, 128, 256};
    float alpha[2] = {1.f, 1.f};
    uint8_t mask[2] = {1, 1};
    void *p = reinterpret_cast<void *>(0x1000), *odd = reinterpret_cast<void *>(0x1008);
    float *o = reinterpret_cast<float *>(p);
    if (mlpmoe_forward_bf16(p, p, p, p, nullptr, alpha, mask, 4, 64, 256, 2, o, nullptr) != MLPMOE_ERR_NULL) ++bad;
    if (mlpmoe_forward_bf16(p, p, p, p, off, alpha, mask, 4, 64, 256, 0, o, nullptr) != MLPMOE_ERR_SHAPE) ++bad;
    if (mlpmoe_forward_bf16(p, p, p, p, off, alpha, mask, 4, 64, 300, 2, o, nullptr) != MLPMOE_ERR_OFFSETS) ++bad;
    if (mlpmoe_forward_bf16(odd, p, p, p, off, alpha, mask, 4, 64, 256, 2, o, nullptr) != MLPMOE_ERR_ALIGN) ++bad;
    if (mlpmoe_forward_f32(nullptr, o, o, o, off, alpha, mask, 4, 64, 256, 2, o, nullptr) != MLPMOE_ERR_NULL) ++bad;
    if (mlpmoe_forward_bf16(p, p, p, p, off, alpha, mask, 0, 64, 256, 2, o, nullptr) != MLPMOE_OK) ++bad;     // T = 0
    if (mlpmoe_forward_bf16_ws(p, p, p, p, off, alpha, mask, 4, 64, 256, 2, o, p, 1 << 20, 99, nullptr) != MLPMOE_ERR_UNSUPPORTED) ++bad;
    if (mlpmoe_forward_bf16_noalloc(p, p, p, p, off, alpha, mask, -1, 64, 256, 2, o, nullptr) != MLPMOE_ERR_SHAPE) ++bad;
    if (mlpmoe_set_workspace(odd, 4096) != MLPMOE_ERR_WORKSPACE) ++bad;
    if (mlpmoe_workspace_bytes(4096, 4096, 14336, 16, 2) < (size_t)4096 * 14336 * 2) ++bad;
    if (mlpmoe_workspace_bytes(1, 1, 1, 65, 2) != 0) ++bad;
    if (mlpmoe_hidden_ld(4870) != 4928) ++bad;
    if (strcmp(mlpmoe_status_string(0), "ok") != 0) ++bad;
    double sp[2] = {0.0, 1.5};
    if (mlpmoe_fade(p, p, off, sp, 64, 256, 2, 2, nullptr, nullptr, nullptr) != MLPMOE_ERR_SHAPE) ++bad;
    int32_t cnt[2] = {1, 200};
    if (mlpmoe_fade_neurons(p, p, off, cnt, 64, 256, 2, 2, mask, nullptr, nullptr) != MLPMOE_ERR_SHAPE) ++bad;
    if (bad) {
        printf("FAILED %d checks\n", bad);
        return 1;
    }
    printf("ok\n");
    return 0;
}
