// Device-side materialisation of the synthetic Chung-Lu graph of fg_inputs/graph.py as an in-neighbour CSR, for runs
// that sample on the device: the same recipe (degree = expected degree rounded up or down at random, every slot an
// independent draw from the power law), evaluated with the device's pow, so a few entries can differ from the host's
// evaluation of the same formula. Whoever uses this CSR treats it as the graph. Input generation only: no step of the
// method under test is in this file.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

struct ChungLu {
    int64_t n;
    uint64_t a, ainv, b;       // rank -> id is (rank * a + b) mod n
    double c, r0, alpha, lo, span, inv_e;
    uint64_t key_deg, key_nbr;
};

__device__ __forceinline__ uint64_t mix64(uint64_t x) {
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}
__device__ __forceinline__ uint64_t word(uint64_t key, uint64_t ctr) { return mix64(key + (ctr + 1ull) * 0x9E3779B97F4A7C15ull); }
__device__ __forceinline__ double unit(uint64_t w) { return (double)(w >> 11) * (1.0 / 9007199254740992.0); }

__global__ void chunglu_degree_kernel(ChungLu G, int64_t* __restrict__ deg) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < G.n; v += stride) {
        const uint64_t n = (uint64_t)G.n;
        const uint64_t rank = (((uint64_t)v + n - G.b) % n) * G.ainv % n;
        const double w = G.c * pow((double)rank + 0.5 + G.r0, -G.alpha);
        const double fl = floor(w);
        deg[v] = (int64_t)fl + (unit(word(G.key_deg, (uint64_t)v)) < (w - fl) ? 1 : 0);
    }
}

__global__ void chunglu_indices_kernel(ChungLu G, const int64_t* __restrict__ indptr, int64_t edges, int32_t* __restrict__ indices) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < edges; e += stride) {
        int64_t lo = 0, hi = G.n;                       // the node whose row holds edge e: indptr[v] <= e < indptr[v + 1]
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (indptr[mid] <= e) lo = mid; else hi = mid;
        }
        const int64_t v = lo, slot = e - indptr[v];
        const double u = unit(word(word(G.key_nbr, (uint64_t)v), (uint64_t)slot));
        double x = floor(pow(G.lo + u * G.span, G.inv_e) - G.r0);
        if (!(x >= 0.0)) x = 0.0;
        if (x > (double)(G.n - 1)) x = (double)(G.n - 1);
        indices[e] = (int32_t)(((uint64_t)x * G.a + G.b) % (uint64_t)G.n);
    }
}

}  // namespace

extern "C" int fgin_chunglu_degrees(int64_t n, uint64_t a, uint64_t ainv, uint64_t b, double c, double r0, double alpha, double lo,
                                    double span, double inv_e, uint64_t key_deg, uint64_t key_nbr, int64_t* deg_out, void* stream) {
    if (n <= 0 || !deg_out) return 1;
    const ChungLu G{n, a, ainv, b, c, r0, alpha, lo, span, inv_e, key_deg, key_nbr};
    hipLaunchKernelGGL(chunglu_degree_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, G, deg_out);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// indptr [n + 1] (device), indices [edges] with edges = indptr[n] known to the caller.
extern "C" int fgin_chunglu_indices(int64_t n, uint64_t a, uint64_t ainv, uint64_t b, double c, double r0, double alpha, double lo,
                                    double span, double inv_e, uint64_t key_deg, uint64_t key_nbr, const int64_t* indptr,
                                    int64_t edges, int32_t* indices_out, void* stream) {
    if (n <= 0 || edges < 0 || !indptr || (edges > 0 && !indices_out)) return 1;
    if (edges == 0) return 0;
    const ChungLu G{n, a, ainv, b, c, r0, alpha, lo, span, inv_e, key_deg, key_nbr};
    hipLaunchKernelGGL(chunglu_indices_kernel, dim3(256 * 32), dim3(256), 0, (hipStream_t)stream, G, indptr, edges, indices_out);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// Synthetic embedding-gradient norms exp(N(0, 1)) keyed by node id (the recipe of fg_inputs/workload.py, grad_norms),
// for loops that sample on the device and so have the node ids only there. Evaluated with the device's log, cos and exp:
// the last bit of a value can differ from the host's evaluation of the same formula.
namespace {
__global__ void grad_norms_kernel(const int32_t* __restrict__ ids, const int64_t* __restrict__ n_dev, int64_t max_n, uint64_t key,
                                  float* __restrict__ out) {
    int64_t n = n_dev ? *n_dev : max_n;
    if (n > max_n) n = max_n;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint64_t c = (uint64_t)(int64_t)ids[i];
    const double u1 = unit(word(key, c * 2ull)), u2 = unit(word(key, c * 2ull + 1ull));
    out[i] = (float)exp(sqrt(-2.0 * log(1.0 - u1)) * cos(6.283185307179586 * u2));
}
}  // namespace

extern "C" int fgin_grad_norms(const int32_t* ids, const int64_t* n_dev, int64_t max_n, uint64_t key, float* out, void* stream) {
    if (max_n < 0 || (max_n > 0 && (!ids || !out))) return 1;
    if (max_n == 0) return 0;
    hipLaunchKernelGGL(grad_norms_kernel, dim3((unsigned)((max_n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, ids, n_dev, max_n,
                       key, out);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
