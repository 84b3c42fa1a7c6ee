/*
 * Seeded synthetic-input helpers shared by the CPU oracle's tests and the GPU
 * tests/bench.  This file builds GRAPHS only (edge lists and their CSC/CSR
 * index arrays); it holds none of the method's arithmetic (no quantization,
 * no GEMM/SPMM/SDDMM, no softmax).
 *
 * R-MAT recipe (Chakrabarti, Zhan, Faloutsos, SDM'04): each edge picks one of
 * four quadrants per address bit with probabilities (a, b, c, d).
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <stdlib.h>

static inline uint64_t mix64(uint64_t z)
{
    /* splitmix64 finalizer (Steele, Lea, Flood 2014) */
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/*
 * Candidate edges number `first` .. `first+count-1` of the stream `seed`.
 * keys[i] = ((uint64)dst << 32) | src after applying `perm` (may be NULL),
 * or UINT64_MAX when the candidate is rejected (endpoint >= n_nodes, or a
 * self pair).  thr = cumulative 16-bit thresholds {a, a+b, a+b+c} * 65536.
 */
void ti_rmat_keys(int scale, uint64_t n_nodes, uint64_t count, uint64_t seed,
                  uint64_t first, const uint32_t *thr, const int32_t *perm,
                  uint64_t *keys)
{
#pragma omp parallel for schedule(static)
    for (int64_t ii = 0; ii < (int64_t)count; ++ii) {
        uint64_t idx = first + (uint64_t)ii;
        uint64_t u = 0, v = 0;
        uint64_t r = 0;
        for (int lvl = 0; lvl < scale; ++lvl) {
            if ((lvl & 3) == 0)
                r = mix64(seed ^ mix64(idx * 16 + (uint64_t)(lvl >> 2)));
            uint32_t t = (uint32_t)(r & 0xffffu);
            r >>= 16;
            unsigned ub, vb;
            if (t < thr[0]) { ub = 0; vb = 0; }
            else if (t < thr[1]) { ub = 0; vb = 1; }
            else if (t < thr[2]) { ub = 1; vb = 0; }
            else { ub = 1; vb = 1; }
            u = (u << 1) | ub;
            v = (v << 1) | vb;
        }
        if (u >= n_nodes || v >= n_nodes || u == v) {
            keys[ii] = UINT64_MAX;
            continue;
        }
        if (perm) { u = (uint64_t)(uint32_t)perm[u]; v = (uint64_t)(uint32_t)perm[v]; }
        keys[ii] = (v << 32) | u;
    }
}

/*
 * In-place compaction of ascending keys: drops repeats and the UINT64_MAX
 * rejection marker; returns the number kept.
 */
int64_t ti_unique_sorted(uint64_t *keys, int64_t n)
{
    int64_t m = 0;
    for (int64_t i = 0; i < n; ++i) {
        uint64_t k = keys[i];
        if (k == UINT64_MAX) break;
        if (m == 0 || keys[m - 1] != k) keys[m++] = k;
    }
    return m;
}

/*
 * Keep exactly `need` of the n keys (order preserved), each subset equally
 * likely: sequential selection sampling (Knuth, TAOCP vol. 2, Algorithm S).
 */
void ti_select(uint64_t *keys, int64_t n, int64_t need, uint64_t seed)
{
    int64_t m = 0;
    for (int64_t i = 0; i < n && m < need; ++i) {
        uint64_t r = mix64(seed ^ mix64((uint64_t)i + 0x5157ull));
        double u = (double)(r >> 11) * (1.0 / 9007199254740992.0);
        if (u * (double)(n - i) < (double)(need - m)) keys[m++] = keys[i];
    }
}

/*
 * Destination-major (CSC) arrays from keys sorted ascending (dst major, src
 * minor): fills in_ptr[n+1] and in_src[nnz].
 */
void ti_csc_from_sorted_keys(int64_t n, int64_t nnz, const uint64_t *keys,
                             int32_t *in_ptr, int32_t *in_src)
{
    memset(in_ptr, 0, (size_t)(n + 1) * sizeof(int32_t));
    for (int64_t e = 0; e < nnz; ++e) {
        in_src[e] = (int32_t)(keys[e] & 0xffffffffu);
        in_ptr[(keys[e] >> 32) + 1] += 1;
    }
    for (int64_t i = 0; i < n; ++i) in_ptr[i + 1] += in_ptr[i];
}

/*
 * Source-major (CSR) view of the same edges.  out_eid[j] is the position of
 * out-edge j in the destination-major order; out lists come out sorted by
 * destination because the input is.
 */
void ti_csr_from_csc(int64_t n, int64_t nnz, const int32_t *in_ptr,
                     const int32_t *in_src, int32_t *out_ptr, int32_t *out_dst,
                     int32_t *out_eid)
{
    memset(out_ptr, 0, (size_t)(n + 1) * sizeof(int32_t));
    for (int64_t e = 0; e < nnz; ++e) out_ptr[in_src[e] + 1] += 1;
    for (int64_t i = 0; i < n; ++i) out_ptr[i + 1] += out_ptr[i];
    int32_t *cur = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    memcpy(cur, out_ptr, (size_t)n * sizeof(int32_t));
    for (int64_t v = 0; v < n; ++v) {
        for (int32_t e = in_ptr[v]; e < in_ptr[v + 1]; ++e) {
            int32_t u = in_src[e];
            int32_t j = cur[u]++;
            out_dst[j] = (int32_t)v;
            out_eid[j] = e;
        }
    }
    free(cur);
}
