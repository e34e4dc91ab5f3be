// Runs the library's host-only entry points (bit allocator, variance alert, size
// helpers) on arrays read from files, for a build of csrc/gact_host.cpp with
// -fsanitize=address,undefined (tests/test_sanitizers.py).
//   host_driver allocate <L> <avg> <n_levels> c.bin numel.bin levels.bin bits.bin
//   host_driver alert    <L> <grad_var> <threshold> c.bin bits.bin out.bin   (out: double ratio, double alert)
//   host_driver sizes    out.bin                                              (a table of size-helper results)
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "gact.h"

static void* slurp(const char* path, size_t bytes) {
    void* p = malloc(bytes ? bytes : 1);      // exactly sized, so that an overrun is seen
    FILE* f = fopen(path, "rb");
    if (!p || !f || fread(p, 1, bytes, f) != bytes) { fprintf(stderr, "cannot read %s\n", path); exit(3); }
    fclose(f);
    return p;
}
static void spill(const char* path, const void* p, size_t bytes) {
    FILE* f = fopen(path, "wb");
    if (!f || fwrite(p, 1, bytes, f) != bytes) { fprintf(stderr, "cannot write %s\n", path); exit(3); }
    fclose(f);
}

int main(int argc, char** argv) {
    if (argc < 2) return 2;
    if (!strcmp(argv[1], "allocate") && argc == 9) {
        const int L = atoi(argv[2]);
        const double avg = atof(argv[3]);
        const int nl = atoi(argv[4]);
        float* c = (float*)slurp(argv[5], (size_t)L * 4);
        int64_t* numel = (int64_t*)slurp(argv[6], (size_t)L * 8);
        int32_t* levels = (int32_t*)slurp(argv[7], (size_t)nl * 4);
        int32_t* bits = (int32_t*)malloc(L ? (size_t)L * 4 : 1);
        const int rc = gact_allocate_bits_levels(c, numel, L, avg, levels, nl, bits);
        if (rc != GACT_OK) { fprintf(stderr, "%s\n", gact_error_string(rc)); return 4; }
        spill(argv[8], bits, (size_t)L * 4);
        free(c); free(numel); free(levels); free(bits);
        return 0;
    }
    if (!strcmp(argv[1], "alert") && argc == 8) {
        const int L = atoi(argv[2]);
        const double gv = atof(argv[3]), thr = atof(argv[4]);
        float* c = (float*)slurp(argv[5], (size_t)L * 4);
        int32_t* bits = (int32_t*)slurp(argv[6], (size_t)L * 4);
        double out[2] = {0.0, 0.0};
        const int rc = gact_variance_alert(c, bits, L, gv, thr, &out[0]);
        if (rc < 0) return 4;
        out[1] = (double)rc;
        spill(argv[7], out, sizeof(out));
        free(c); free(bits);
        return 0;
    }
    if (!strcmp(argv[1], "sizes") && argc == 3) {
        std::vector<uint64_t> out;
        const int64_t ns[] = {-1, 0, 1, 7, 8, 31, 32, 127, 128, 129, 1000, 2048, 1 << 20, (1ll << 33) + 5};
        for (int64_t n : ns) {
            for (int b : {1, 2, 4, 8}) out.push_back((uint64_t)gact_packed_bytes(n, b));
            for (int G : {32, 96, 128, 256, 1024}) out.push_back((uint64_t)gact_num_groups(n, G));
        }
        spill(argv[2], out.data(), out.size() * 8);
        return 0;
    }
    fprintf(stderr, "bad command line\n");
    return 2;
}
