// A reasonable multi-core CPU implementation of one compression call (error feedback + exact Top-k by
// std::nth_element on a copy of the keys + one selection sweep), timed by bench.py next to the GPU path and next
// to the oracle.  BASELINE ONLY: it is neither the oracle (which is a plain full sort) nor part of the library,
// it checks nothing and nothing is checked against it.
//
// Build: g++ -O2 -fopenmp -shared -fPIC bench_cpu_select.cpp -o libbench_cpu_select.so
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <functional>
#include <vector>

#include <omp.h>

extern "C" {

// acc = residual + grad in place, select the k largest |acc| (ties by lower index), write the message in
// ascending index order, zero the selected residual slots, return ||selected||^2 / ||acc||^2.
// Returns the number of threads used in *threads.
double cpu_select_compress(const float* grad, float* residual, int64_t n, int64_t k, int32_t* out_idx, float* out_val,
                           int* threads)
{
    std::vector<uint32_t> key((size_t)n);
    double ss_all = 0.0;
    *threads = omp_get_max_threads();
#pragma omp parallel for reduction(+ : ss_all) schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const float a = residual[i] + grad[i];
        residual[i] = a;
        uint32_t u;
        std::memcpy(&u, &a, 4);
        key[(size_t)i] = u & 0x7FFFFFFFu;
        ss_all += (double)a * (double)a;
    }
    std::vector<uint32_t> work(key);
    std::nth_element(work.begin(), work.begin() + (k - 1), work.end(), std::greater<uint32_t>());
    const uint32_t tau = work[(size_t)(k - 1)];
    int64_t above = 0;
#pragma omp parallel for reduction(+ : above) schedule(static)
    for (int64_t i = 0; i < n; ++i) above += key[(size_t)i] > tau;
    int64_t need = k - above, at = 0;  // ties taken in index order
    double ss_sel = 0.0;
    for (int64_t i = 0; i < n; ++i) {   // ordered compaction (sequential: the output order is the index order)
        const uint32_t m = key[(size_t)i];
        bool take = m > tau;
        if (m == tau && need > 0) { take = true; --need; }
        if (take) {
            out_idx[at] = (int32_t)i;
            out_val[at] = residual[i];
            ss_sel += (double)residual[i] * (double)residual[i];
            residual[i] = 0.0f;
            ++at;
        }
    }
    return ss_all == 0.0 ? 1.0 : ss_sel / ss_all;
}

}  // extern "C"
