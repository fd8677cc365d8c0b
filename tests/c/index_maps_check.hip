// Host-only check of the index maps the fused kernels' offline weight and bias packing relies on
// (compiled with hipcc because the header also holds device code; nothing here touches a GPU).
#include <stdio.h>
#include <string.h>

#include "dhq_fused_common.h"

static int is_permutation(const int *v, int n)
{
    static unsigned char seen[512];
    memset(seen, 0, sizeof(seen));
    for (int i = 0; i < n; ++i) {
        if (v[i] < 0 || v[i] >= n || seen[v[i]]) return 0;
        seen[v[i]] = 1;
    }
    return 1;
}

int main()
{
    const int widths[] = {32, 64, 128, 256, 512};
    for (int w = 0; w < 5; ++w) {
        const int NF = widths[w], NR = NF / 2;
        int a[512], b[512], c[512];
        for (int u = 0; u < 2; ++u)
            for (int s = 0; s < NR; ++s) {
                a[u * NR + s] = hm_index(s, u);
                b[u * NR + s] = rot_index(s, u);
                // the accumulator layout of a 32 x 32 MFMA: register 16 T + 4 g + e of lane half u is row 8 g + 4 u + e of tile T
                const int T = s >> 4, g = (s >> 2) & 3, e = s & 3;
                if (hm_index(s, u) != 32 * T + 8 * g + 4 * u + e) { printf("hm_index(%d, %d)\n", s, u); return 1; }
                // the lane swap exchanges the roles of bit 0 of s and of u
                if (rot_index(s, u) != hm_index((s & ~1) | u, s & 1)) { printf("rot_index(%d, %d)\n", s, u); return 1; }
            }
        if (!is_permutation(a, NF) || !is_permutation(b, NF)) { printf("not a permutation at width %d\n", NF); return 1; }
        for (int f = 0; f < NF; ++f) c[f] = bias_slot(f);
        if (!is_permutation(c, NF)) { printf("bias_slot is not a permutation at width %d\n", NF); return 1; }
        for (int f = 0; f < NF; f += 4)
            for (int e = 1; e < 4; ++e)
                if (bias_slot(f + e) != bias_slot(f) + e) { printf("bias_slot(%d)\n", f + e); return 1; }
        // a lane half reads the four biases of rows 8 g + 4 u .. + 3 of tile T as one float4 at index (T * 4 + g) * 2 + u
        for (int f = 0; f < NF; f += 4) {
            const int T = f >> 5, g = (f >> 3) & 3, u = (f >> 2) & 1;
            if (bias_slot(f) != 4 * ((T * 4 + g) * 2 + u)) { printf("bias_slot group %d\n", f); return 1; }
        }
    }
    printf("index_maps ok\n");
    return 0;
}
