/*
 * A plain C99 client of the library: shows that include/zi.h is a C header (no C++ needed), prints the
 * struct sizes the Python binding must agree with, and drives the calls that need no GPU.
 * Output: one "key value..." line per fact; tests/test_abi_c_client.py reads them.
 */
#include <stdio.h>
#include <string.h>

#include "zi.h"

int main(void)
{
    printf("sizeof_norm_result %zu\n", sizeof(zi_norm_result));
    printf("sizeof_tensor %zu\n", sizeof(zi_tensor));
    printf("sizeof_config %zu\n", sizeof(zi_adamw_config));
    printf("sizeof_segment %zu\n", sizeof(zi_chunk_segment));
    printf("sizeof_stats %zu\n", sizeof(zi_stream_stats));
    printf("sizeof_file_tensor %zu\n", sizeof(zi_file_tensor));
    printf("workspace %zu\n", zi_norm_workspace_bytes(1000, 1));

    /* chunk plan: one tensor of two and a half chunks and one small tensor */
    const int64_t numel[2] = {2 * 4096 + 2048, 100};
    zi_chunk_segment seg[8];
    int64_t n_seg = 0, n_use = 0;
    zi_status st = zi_plan_chunks(numel, 2, 4096, seg, 8, &n_seg, &n_use);
    printf("plan %d %lld %lld\n", (int)st, (long long)n_seg, (long long)n_use);
    for (int64_t i = 0; i < n_seg && i < 8; ++i)
        printf("segment %d %lld %lld %lld %lld\n", seg[i].tensor, (long long)seg[i].elem_offset,
               (long long)seg[i].count, (long long)seg[i].slot_use, (long long)seg[i].slot_offset);

    /* argument errors come back as codes with a text, nothing aborts */
    zi_adamw_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.lr = 1e-3f; cfg.beta1 = 0.9f; cfg.beta2 = 0.999f; cfg.eps = 1e-8f; cfg.weight_decay = 0.01f;
    cfg.step = 0; cfg.loss_scale = 1.0f; cfg.max_grad_norm = 0.0f; cfg.mode = ZI_MODE_ADAMW;
    st = zi_adamw_step(NULL, 0, ZI_BF16, &cfg, NULL, NULL);
    printf("bad_step %d %s\n", (int)st, zi_last_error()[0] ? "text" : "notext");
    cfg.step = 1;
    st = zi_adamw_step(NULL, 0, ZI_BF16, &cfg, NULL, NULL);     /* empty list: valid, does nothing */
    printf("empty_list %d\n", (int)st);

    /* the host-CPU step on eight elements (bf16 gradients of 2^-10, first step) */
    float p[8], m[8], v[8];
    uint16_t g[8], lp[8];
    for (int i = 0; i < 8; ++i) { p[i] = 0.5f + 0.125f * (float)i; m[i] = 0.0f; v[i] = 0.0f; g[i] = 0x3A80; lp[i] = 0; }
    zi_tensor t;
    t.p = p; t.m = m; t.v = v; t.g = g; t.p_lp = lp; t.numel = 8;
    zi_norm_result nr;
    st = zi_host_grad_norm(&t, 1, ZI_BF16, 1.0f, &nr, 2);
    printf("host_norm %d %.17g %.17g %u\n", (int)st, nr.sumsq, nr.norm, nr.found_inf);
    st = zi_host_adamw_step(&t, 1, ZI_BF16, &cfg, &nr, 2);
    printf("host_step %d\n", (int)st);
    for (int i = 0; i < 8; ++i) {
        uint32_t pb, mb, vb;
        memcpy(&pb, &p[i], 4); memcpy(&mb, &m[i], 4); memcpy(&vb, &v[i], 4);
        printf("element %d %u %u %u %u\n", i, pb, mb, vb, (unsigned)lp[i]);
    }
    return 0;
}
