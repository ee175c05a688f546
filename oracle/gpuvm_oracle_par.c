/*
 * All-host-cores leg of the CPU baseline.  TEST / BENCHMARK INFRASTRUCTURE ONLY.
 *
 * The five stated workloads computed directly on host memory, as in Part 1 of
 * gpuvm_oracle.c, with the outermost loop handed to all cores by a plain
 * OpenMP parallel-for - no blocking, no tuning.  It exists only so that the
 * benchmark can put "what the box's CPU does with every core" beside the GPU
 * path; the expected values of every parity test come from the sequential
 * oracle, never from here.  The CPU suite checks that each function here
 * returns what its sequential counterpart returns.  Shares no code with the
 * HIP library and must never be linked into or called from the product path.
 */
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>

int par_threads(void) { return omp_get_max_threads(); }

/* out[k] = host[idx[k]], sum = sum_k out[k] */
void par_gather(const uint32_t *host, const uint32_t *idx, uint64_t n, uint32_t *out, uint64_t *sum)
{
    uint64_t s = 0;
#pragma omp parallel for reduction(+ : s) schedule(static)
    for (int64_t k = 0; k < (int64_t)n; ++k) {
        out[k] = host[idx[k]];
        s += (uint64_t)out[k];
    }
    *sum = s;
}

/* fp64 sum of every block of block_elems consecutive floats, index order inside a block */
void par_stream_reduce(const float *x, uint64_t n, uint64_t block_elems, int passes, double *s)
{
    int64_t nblocks = (int64_t)((n + block_elems - 1) / block_elems);
    for (int p = 0; p < passes; ++p) {
#pragma omp parallel for schedule(static)
        for (int64_t b = 0; b < nblocks; ++b) {
            uint64_t lo = (uint64_t)b * block_elems;
            uint64_t hi = lo + block_elems < n ? lo + block_elems : n;
            double acc = 0.0;
            for (uint64_t i = lo; i < hi; ++i) acc += (double)x[i];
            s[(uint64_t)p * (uint64_t)nblocks + (uint64_t)b] = acc;
        }
    }
}

/* hop distance from src, -1 = unreachable: one sweep over all vertices per level */
int par_bfs(const int64_t *row_ptr, const int32_t *col_idx, int64_t nv, int64_t src, int32_t *level)
{
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < nv; ++v) level[v] = -1;
    level[src] = 0;
    for (int32_t cur = 0;; ++cur) {
        int found = 0;
#pragma omp parallel for schedule(dynamic, 4096) reduction(| : found)
        for (int64_t v = 0; v < nv; ++v) {
            if (level[v] != cur) continue;
            for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
                int32_t u = col_idx[e];
                int32_t lu;
#pragma omp atomic read
                lu = level[u];
                if (lu < 0) {
                    /* several threads may store the same value */
#pragma omp atomic write
                    level[u] = cur + 1;
                    found = 1;
                }
            }
        }
        if (!found) break;
    }
    return 0;
}

/* bags summed in listed order in fp32, one rounding per add */
void par_embedding_bag_f32(const float *table, uint64_t dim, const int32_t *ids, uint64_t bags,
                           uint64_t bag_len, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < (int64_t)bags; ++b)
        for (uint64_t c = 0; c < dim; ++c) {
            volatile float acc = 0.0f;
            for (uint64_t j = 0; j < bag_len; ++j)
                acc = acc + table[(uint64_t)ids[(uint64_t)b * bag_len + j] * dim + c];
            out[(uint64_t)b * dim + c] = acc;
        }
}

/* host[idx[k]] += 1, concurrent updates of one element made atomic */
void par_scatter_increment(uint64_t *host, const uint32_t *idx, uint64_t k)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)k; ++i) {
#pragma omp atomic update
        host[idx[i]] += 1;
    }
}
