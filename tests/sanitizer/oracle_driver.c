/* Runs the CPU oracle's entry points on arrays read from files, for a build of
 * oracle/gact_oracle.c with -fsanitize=address,undefined (tests/test_sanitizers.py).
 * Test infrastructure: no arithmetic of the method lives here.
 *
 *   oracle_driver compress   <dtype> <n> <G> <bits> <seed> x.bin packed.bin gmin.bin gscale.bin y.bin
 *   oracle_driver allocate   <L> <avg> <n_levels> c.bin numel.bin levels.bin bits.bin
 *   oracle_driver footprint  <dtype> <n> <n_samples> x.bin out.bin
 *   oracle_driver sensitivity <dtype> <n> <bits> g0.bin g1.bin out.bin
 * Exit status 0 = the oracle returned 0 and every file was read and written in full.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int64_t gact_oracle_num_groups(int64_t n, int group_size);
int64_t gact_oracle_packed_bytes(int64_t n, int bits);
int gact_oracle_compress(const void *x, int dtype, int64_t n, int group_size, int bits, uint64_t seed,
                         uint8_t *packed, float *gmin, float *gscale);
int gact_oracle_decompress(const uint8_t *packed, const float *gmin, const float *gscale, int64_t n,
                           int group_size, int bits, void *y, int dtype);
int gact_oracle_allocate_bits_levels(const float *sensitivity, const int64_t *numel, int L, double avg,
                                     const int32_t *levels, int n_levels, int32_t *bits_out);
int gact_oracle_footprint(const void *x, int64_t n, int dtype, int n_samples, double *out);
int gact_oracle_sensitivity(const void *const *g0, const void *const *g1, const int64_t *n, const int *dtype,
                            int K, int bits, double *out);

static void *slurp(const char *path, size_t bytes) {
    /* exactly `bytes` bytes, in a block of exactly that size so that an overrun is seen */
    void *p = malloc(bytes ? bytes : 1);
    FILE *f = fopen(path, "rb");
    if (!p || !f || fread(p, 1, bytes, f) != bytes) { fprintf(stderr, "cannot read %s\n", path); exit(3); }
    fclose(f);
    return p;
}
static void spill(const char *path, const void *p, size_t bytes) {
    FILE *f = fopen(path, "wb");
    if (!f || fwrite(p, 1, bytes, f) != bytes) { fprintf(stderr, "cannot write %s\n", path); exit(3); }
    fclose(f);
}

int main(int argc, char **argv) {
    if (argc < 2) return 2;
    if (!strcmp(argv[1], "compress") && argc == 12) {
        const int dtype = atoi(argv[2]);
        const int64_t n = atoll(argv[3]);
        const int G = atoi(argv[4]), bits = atoi(argv[5]);
        const uint64_t seed = strtoull(argv[6], NULL, 10);
        const size_t es = dtype ? 2 : 4;
        const size_t ng = (size_t)gact_oracle_num_groups(n, G), pb = (size_t)gact_oracle_packed_bytes(n, bits);
        void *x = slurp(argv[7], (size_t)n * es);
        uint8_t *packed = malloc(pb ? pb : 1);
        float *gmin = malloc(ng ? ng * 4 : 1), *gscale = malloc(ng ? ng * 4 : 1);
        void *y = malloc(n ? (size_t)n * es : 1);
        if (gact_oracle_compress(x, dtype, n, G, bits, seed, packed, gmin, gscale)) return 4;
        if (gact_oracle_decompress(packed, gmin, gscale, n, G, bits, y, dtype)) return 5;
        spill(argv[8], packed, pb); spill(argv[9], gmin, ng * 4); spill(argv[10], gscale, ng * 4);
        spill(argv[11], y, (size_t)n * es);
        free(x); free(packed); free(gmin); free(gscale); free(y);
        return 0;
    }
    if (!strcmp(argv[1], "allocate") && argc == 9) {
        const int L = atoi(argv[2]);
        const double avg = atof(argv[3]);
        const int nl = atoi(argv[4]);
        float *c = slurp(argv[5], (size_t)L * 4);
        int64_t *numel = slurp(argv[6], (size_t)L * 8);
        int32_t *levels = slurp(argv[7], (size_t)nl * 4);
        int32_t *bits = malloc(L ? (size_t)L * 4 : 1);
        if (gact_oracle_allocate_bits_levels(c, numel, L, avg, levels, nl, bits)) return 4;
        spill(argv[8], bits, (size_t)L * 4);
        free(c); free(numel); free(levels); free(bits);
        return 0;
    }
    if (!strcmp(argv[1], "footprint") && argc == 7) {
        const int dtype = atoi(argv[2]);
        const int64_t n = atoll(argv[3]);
        const int ns = atoi(argv[4]);
        void *x = slurp(argv[5], (size_t)n * (dtype ? 2 : 4));
        double *out = malloc((size_t)(1 + ns) * 8);
        if (gact_oracle_footprint(x, n, dtype, ns, out)) return 4;
        spill(argv[6], out, (size_t)(1 + ns) * 8);
        free(x); free(out);
        return 0;
    }
    if (!strcmp(argv[1], "sensitivity") && argc == 8) {
        const int dtype = atoi(argv[2]);
        const int64_t n = atoll(argv[3]);
        const int bits = atoi(argv[4]);
        const void *g0 = slurp(argv[5], (size_t)n * (dtype ? 2 : 4));
        const void *g1 = slurp(argv[6], (size_t)n * (dtype ? 2 : 4));
        double out = 0.0;
        if (gact_oracle_sensitivity(&g0, &g1, &n, &dtype, 1, bits, &out)) return 4;
        spill(argv[7], &out, 8);
        free((void *)g0); free((void *)g1);
        return 0;
    }
    fprintf(stderr, "bad command line\n");
    return 2;
}
