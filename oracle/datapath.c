/*
 * CPU oracle for the merged-gradient data path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain element loops written from the paper's definitions.  It shares no code
 * with the HIP library and must never be linked or called by the product path
 * (only tests, the smoke check and the benchmark's cpu_baseline leg use it).
 * Build with -ffp-contract=off so that every fp32 operation is rounded once.
 *
 * All pointers are host pointers.  Layers are 0-based here (index 0 = the
 * paper's layer 1).  A "group" is a list of layer indices in arrival order of
 * the backward pass, highest layer first (Algorithm 2 pushes l = L..1 into the
 * layer buffer and sends it when a non-merged layer arrives).
 *
 *   oracle_pack      Algorithm 2's layer buffer: the group's gradients laid end
 *                    to end, in arrival order, no padding (Condition 3: the merged
 *                    message has p(l-1)+p(l) parameters, nothing more).
 *   oracle_reduce    Eq. 2: (1/N) * sum over workers g of the gradient; workers
 *                    are added in order 0..N-1 in fp32 and the sum is multiplied
 *                    by the fp32 reciprocal of N.
 *   oracle_unpack    the inverse of pack for one buffer.
 *   oracle_sgd       Eq. 1 / Algorithm 2's W = W - eta * grad, extended with a
 *                    momentum buffer: v = mu*v + g ; w = w - eta*v.  With mu = 0
 *                    it is exactly the paper's update.
 *
 * `threads` > 1 splits the element loop of the current layer (pack, unpack) or of
 * the whole buffer (reduce, update) statically over that many OpenMP threads;
 * each element is still produced by the same sequence of operations.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Copy the group's layers of one replica into `merged`, bit for bit.
 * grads[l] points at layer l; p[l] is its element count. */
void oracle_pack(const uint32_t *const *grads, const uint64_t *p,
                 const int32_t *group_layers, int32_t n_group_layers,
                 uint32_t *merged, int32_t threads)
{
    uint64_t off = 0;
    (void)threads;
    for (int32_t k = 0; k < n_group_layers; ++k) {
        int32_t l = group_layers[k];
        int64_t n = (int64_t)p[l];
#pragma omp parallel for schedule(static) num_threads(threads) if (threads > 1 && n > 32768)
        for (int64_t i = 0; i < n; ++i)
            merged[off + (uint64_t)i] = grads[l][i];
        off += p[l];
    }
}

/* out[j] = (((x0[j] + x1[j]) + x2[j]) + ... + x{N-1}[j]) * (1.0f / N) */
void oracle_reduce(const float *const *x, int32_t n_workers, uint64_t n_elems,
                   float *out, int32_t threads)
{
    const float inv_n = 1.0f / (float)n_workers;
    int64_t n = (int64_t)n_elems;
    (void)threads;
#pragma omp parallel for schedule(static) num_threads(threads) if (threads > 1)
    for (int64_t j = 0; j < n; ++j) {
        float acc = x[0][j];
        for (int32_t g = 1; g < n_workers; ++g)
            acc = acc + x[g][j];
        out[j] = acc * inv_n;
    }
}

/* Scatter one merged buffer back to the group's per-layer tensors, bit for bit. */
void oracle_unpack(const uint32_t *merged, const uint64_t *p,
                   const int32_t *group_layers, int32_t n_group_layers,
                   uint32_t *const *out, int32_t threads)
{
    uint64_t off = 0;
    (void)threads;
    for (int32_t k = 0; k < n_group_layers; ++k) {
        int32_t l = group_layers[k];
        int64_t n = (int64_t)p[l];
#pragma omp parallel for schedule(static) num_threads(threads) if (threads > 1 && n > 32768)
        for (int64_t i = 0; i < n; ++i)
            out[l][i] = merged[off + (uint64_t)i];
        off += p[l];
    }
}

/* v = mu*v + g ; w = w - lr*v, every operation rounded to fp32 on its own. */
void oracle_sgd(float *w, float *v, const float *g, uint64_t n_elems,
                float lr, float mu, int32_t threads)
{
    int64_t n = (int64_t)n_elems;
    (void)threads;
#pragma omp parallel for schedule(static) num_threads(threads) if (threads > 1)
    for (int64_t i = 0; i < n; ++i) {
        float mv = mu * v[i];
        float vn = mv + g[i];
        float step = lr * vn;
        v[i] = vn;
        w[i] = w[i] - step;
    }
}

int32_t oracle_max_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}
