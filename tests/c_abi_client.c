/* A plain C99 client of the library's C ABI (compiled and run by tests/test_c_abi_client.py):
 * rearrange and order the filters of a small 1x1 layer, prune it, pack it on the host only, read
 * the canonical arrays and the layout figures back. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sbn.h"

int main(void)
{
    enum { N = 16, K = 24, GO = 4, GI = 4 };
    float w[N * K], bias[N];
    uint8_t mask[(N / GO) * (K / GI)];
    unsigned s = 12345u;
    for (int i = 0; i < N * K; ++i) {
        s = s * 1664525u + 1013904223u;
        w[i] = (float)(s >> 8) / 16777216.0f - 0.5f;
    }
    for (int i = 0; i < N; ++i) bias[i] = 0.01f * (float)i;
    {
        /* offline steps on the original weights: which filters share a group, then the groups' order */
        sbn_layer_desc_t l;
        int32_t perm[N], *perms[1];
        const int parent[1] = {-1};
        int seen[N];
        memset(&l, 0, sizeof l);
        l.kind = SBN_CONV1X1, l.c_in = K, l.c_out = N, l.go = GO, l.gi = GI, l.stride = 1, l.w = w;
        perms[0] = perm;
        if (sbn_rearrange(&l, 1, parent, NULL, 50, 7u, 200, perms) != SBN_OK ||
            sbn_order_groups(&l, 1, parent, NULL, 50, perms) != SBN_OK) {
            fprintf(stderr, "rearrange: %s\n", sbn_last_error());
            return 1;
        }
        memset(seen, 0, sizeof seen);
        for (int i = 0; i < N; ++i) {
            if (perm[i] < 0 || perm[i] >= N || seen[perm[i]]++) return 1;
        }
    }
    if (sbn_prune_magnitude(w, SBN_CONV1X1, K, N, GO, GI, 50, mask) != SBN_OK) {
        fprintf(stderr, "prune: %s\n", sbn_last_error());
        return 1;
    }
    int kept = 0;
    for (size_t i = 0; i < sizeof mask; ++i) kept += mask[i];
    sbn_layer_desc_t d;
    memset(&d, 0, sizeof d);
    d.kind = SBN_CONV1X1, d.c_in = K, d.c_out = N, d.go = GO, d.gi = GI, d.stride = 1;
    d.w = w, d.mask = mask, d.bias = bias, d.act = SBN_ACT_RELU;
    sbn_packed_t* p = NULL;
    if (sbn_pack(&d, -1, &p) != SBN_OK || !p) {
        fprintf(stderr, "pack: %s\n", sbn_last_error());
        return 1;
    }
    size_t nnz = 0;
    uint32_t row_ptr[N / GO + 1];
    if (sbn_export(p, row_ptr, NULL, NULL, NULL, NULL, NULL, &nnz) != SBN_OK || (int)nnz != kept ||
        row_ptr[N / GO] != nnz) {
        fprintf(stderr, "export: %s\n", sbn_last_error());
        return 1;
    }
    {
        size_t entries = 0, bytes = 0;
        int every_piece = -1;
        if (sbn_packed_layout(p, &entries, &bytes, &every_piece) != SBN_OK || entries == 0 || entries > (size_t)(K / 4) ||
            bytes == 0 || every_piece != 0)                 /* one bundle of 16 filters; a single chunk has no every-piece tables */
            return 1;
    }
    if (sbn_conv1x1_sparse(p, w, bias, 1, 1, 1, NULL) != SBN_ENODEV) return 1;   /* no device copy: refused */
    if (sbn_pack(&d, -1, NULL) != SBN_EINVAL || strlen(sbn_last_error()) == 0) return 1;
    sbn_free(p);
    printf("c client ok: %d of %d blocks kept\n", kept, (int)sizeof mask);
    return 0;
}
