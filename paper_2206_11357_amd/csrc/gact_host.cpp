// Entry points of the C ABI (include/gact.h) that run on the host alone and use
// nothing of the HIP runtime: buffer sizes, error names, the bit allocator
// (Eq. (ilp) of arXiv 2206.11357, Sec. 4.1, solved by greedy descent with a
// binary heap) and the variance alert of Sec. 4.2.  Kept apart from the launch
// code so that it also builds with a plain host compiler (for sanitizer runs).
#include <cmath>
#include <cstdint>
#include <queue>
#include <vector>

#include "gact.h"

namespace {
bool bits_ok(int bits) { return bits == 1 || bits == 2 || bits == 4 || bits == 8; }
}  // namespace

extern "C" {

size_t gact_num_groups(int64_t n, int group_size) {
    if (n <= 0 || group_size <= 0) return 0;
    return (size_t)((n + group_size - 1) / group_size);
}

size_t gact_packed_bytes(int64_t n, int bits) {
    if (n <= 0 || bits <= 0) return 0;
    const uint64_t bytes = ((uint64_t)n * (uint64_t)bits + 7) / 8;
    return (size_t)((bytes + 15) / 16 * 16);
}

const char* gact_error_string(int code) {
    switch (code) {
        case GACT_OK: return "ok";
        case GACT_E_ARG: return "bad argument (null/misaligned pointer, negative size, bad dtype, small workspace)";
        case GACT_E_BITS: return "bits must be 1, 2, 4 or 8";
        case GACT_E_GROUP: return "group_size must be a multiple of 32 in [32, 1024]";
        case GACT_E_BUDGET: return "avg_bit_budget must be >= 1";
        case GACT_E_HIP: return "HIP runtime error";
        case GACT_E_CAPTURE: return "the stream is capturing a HIP graph and this call needs a table upload from host memory";
        case GACT_E_SCRATCH: return "the tensor needs more than the library's static scratch area (GACT_NOALLOC_SCRATCH_BYTES)";
        default: return "unknown error";
    }
}

int gact_variance_alert(const float* h_sensitivity, const int32_t* h_bits, int L, double grad_var,
                        double threshold, double* h_ratio) {
    if (L < 0 || (L > 0 && (!h_sensitivity || !h_bits)) || !(grad_var > 0.0)) return GACT_E_ARG;
    double V = 0.0;
    for (int l = 0; l < L; ++l) {
        // 32: a tensor the allocator left uncompressed; it adds c_l (2^32 - 1)^-2
        if (!bits_ok(h_bits[l]) && h_bits[l] != GACT_BITS_UNCOMPRESSED) return GACT_E_BITS;
        if (!(h_sensitivity[l] >= 0.0f) || std::isinf(h_sensitivity[l])) return GACT_E_ARG;
        const double B = std::ldexp(1.0, h_bits[l]) - 1.0;
        V += (double)h_sensitivity[l] / (B * B);
    }
    const double ratio = V / grad_var;
    if (h_ratio) *h_ratio = ratio;
    return ratio > threshold ? 1 : 0;
}

// ---------------------------------------------------------------- allocator
int gact_allocate_bits_levels(const float* h_sensitivity, const int64_t* h_numel, int L,
                              double avg_bit_budget, const int32_t* h_levels, int n_levels,
                              int32_t* h_bits_out) {
    if (L < 0 || n_levels < 1 || n_levels > 5 || !h_levels) return GACT_E_ARG;
    int level[5];
    double S[5];
    for (int k = 0; k < n_levels; ++k) {
        const int b = h_levels[k];
        if (!(bits_ok(b) || b == GACT_BITS_UNCOMPRESSED)) return GACT_E_BITS;
        if (k > 0 && b <= level[k - 1]) return GACT_E_BITS;
        level[k] = b;
        const double B = std::ldexp(1.0, b) - 1.0;
        S[k] = 1.0 / (B * B);
    }
    if (!(avg_bit_budget >= (double)level[0])) return GACT_E_BUDGET;
    if (L == 0) return GACT_OK;
    if (!h_sensitivity || !h_numel || !h_bits_out) return GACT_E_ARG;

    const int top = n_levels - 1;
    uint64_t total = 0;
    for (int l = 0; l < L; ++l) {
        const double c = (double)h_sensitivity[l];
        if (!(c >= 0.0) || std::isinf(c) || h_numel[l] < 0) return GACT_E_ARG;
        total += (uint64_t)h_numel[l];
    }
    const double cap = std::floor(avg_bit_budget * (double)total);
    const uint64_t budget = cap >= 18446744073709549568.0 ? UINT64_MAX : (uint64_t)cap;
    uint64_t used = (uint64_t)level[top] * total;

    // cost of moving tensor l from level index k to k-1: variance added per bit saved
    auto step_key = [&](int l, int k) {
        return ((double)h_sensitivity[l] * (S[k - 1] - S[k])) /
               ((double)h_numel[l] * (double)(level[k] - level[k - 1]));
    };
    struct Step { double key; int l; };
    struct Later {   // min-heap on (key, l)
        bool operator()(const Step& a, const Step& b) const {
            return a.key > b.key || (a.key == b.key && a.l > b.l);
        }
    };
    std::vector<int> idx((size_t)L, top);
    std::priority_queue<Step, std::vector<Step>, Later> heap;
    for (int l = 0; l < L; ++l) {
        h_bits_out[l] = level[top];
        if (h_numel[l] > 0 && top > 0) heap.push(Step{step_key(l, top), l});
    }
    while (used > budget && !heap.empty()) {
        const Step s = heap.top();
        heap.pop();
        const int k = idx[(size_t)s.l];
        used -= (uint64_t)h_numel[s.l] * (uint64_t)(level[k] - level[k - 1]);
        idx[(size_t)s.l] = k - 1;
        h_bits_out[s.l] = level[k - 1];
        if (k - 1 > 0) heap.push(Step{step_key(s.l, k - 1), s.l});
    }
    return GACT_OK;
}

int gact_allocate_bits(const float* h_sensitivity, const int64_t* h_numel, int L,
                       double avg_bit_budget, int32_t* h_bits_out) {
    static const int32_t levels[4] = {1, 2, 4, 8};
    return gact_allocate_bits_levels(h_sensitivity, h_numel, L, avg_bit_budget, levels, 4,
                                     h_bits_out);
}

}  // extern "C"
