/*
 * CPU oracle for the mini-batch GCN hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain statement of what the path computes.  It is used by the tests,
 * by the smoke check and by the benchmark's cpu_baseline leg, and by nothing else; the product
 * (the HIP library) never links, loads or calls it, and the two share no code.
 *
 * Every function follows one passage of the paper (ScaleGNN, arXiv 2604.02651):
 *   oracle_sample_uniform   Sec. III-D "Vertex Sampling", Eq. 20  (uniform B-subset of V)
 *   oracle_induced_csr      Sec. III-D Eq. 21 (induced edges), Eqs. 23-24 (p and the rescale),
 *                           Sec. II-A Eq. 3 (symmetric normalisation of A + I)
 *   oracle_induced_csr_range   Algorithm 2 with its row and column ranges (one shard of that matrix)
 *   oracle_gather_rows      Sec. III-D Eq. 26 (feature / label slicing)
 *   oracle_spmm, oracle_gemm, oracle_gcn_fwd   Sec. III-B Eqs. 5-6 (+ ReLU, Eq. 8)
 *   oracle_gcn_bwd          Sec. III-C, the three layer-backward equations (grad W, grad H_agg,
 *                           transposed SpMM)
 *   oracle_softmax_xent     Sec. III-B "Output Head and Loss" (cross-entropy, single label)
 *   oracle_tail_fwd/_bwd    Sec. III-B Eqs. 7-10 (RMSNorm with a learnable scale, ReLU, dropout,
 *                           residual add) and the element-wise part of Sec. III-C
 *   oracle_dropout_keep     the dropout mask M_drop of Eq. 9 (see below)
 * The random generator is not the paper's (it uses a framework permutation whose stream is not
 * reproducible).  The sample is pinned instead as: the B vertices with the smallest
 * (key(v), v), where key(v) is 64 bits of Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11)
 * keyed by the seed and counted by (v / 2, step).  Any exact selection of that set is uniform
 * over B-subsets whenever keys are distinct, which is what Eq. 20 asks for.
 *
 * Dropout (Eq. 9) needs random numbers too.  The mask is pinned as: element e = i * d + j of
 * layer l at step t is kept iff word (e mod 4) of Philox4x32-10 with key = (seed lo, seed hi) and
 * counter = (e / 4 lo, e / 4 hi, t mod 2^32, 2^31 + l) is >= floor(q * 2^32); kept elements are
 * scaled by 1 / (1 - q) (the paper only says a fraction is zeroed; the scaling that keeps the
 * expectation is the reading taken).  RMSNorm: n = gamma * z / sqrt(mean(z^2) + eps); the paper's
 * RMS has no eps (eps = 0 gives its formula exactly).
 *
 * All floating-point work is done in double precision.  Values that the method stores in fp32
 * (edge weights) are rounded to fp32 once, where the definition says they are stored.
 *
 * Parity pins (tests/, marker "not gpu"): Philox against the published known-answer vectors and a
 * big-integer Python version; the sampler against an independent threshold selection and the
 * inclusion-probability statistics of Eq. 20; the induced CSR against dense brute force, scipy
 * slicing, a literal walk through Algorithm 2's phases and the exact enumeration of Eq. 25; the
 * layer against dense numpy, torch autograd and central finite differences; the shards of Algorithm 2
 * by tiling against the full matrix; the layer tail against closed forms, its invariances, an independent
 * evaluation of the dropout counter mapping, torch autograd and finite differences.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------------------------ */
/* Philox4x32-10                                                                                */
/* ------------------------------------------------------------------------------------------ */

#define PHILOX_M0 0xD2511F53u
#define PHILOX_M1 0xCD9E8D57u
#define PHILOX_W0 0x9E3779B9u
#define PHILOX_W1 0xBB67AE85u

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)PHILOX_M0 * c0;
        uint64_t p1 = (uint64_t)PHILOX_M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += PHILOX_W0;
        k1 += PHILOX_W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* 64-bit selection key of vertex v at a given step: vertices 2j and 2j+1 share Philox block j;
 * the even vertex takes words (1,0), the odd vertex words (3,2), high word first. */
uint64_t oracle_vertex_key(uint64_t seed, uint64_t step, uint64_t v)
{
    uint64_t j = v >> 1;
    uint32_t ctr[4] = { (uint32_t)j, (uint32_t)(j >> 32), (uint32_t)step, (uint32_t)(step >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    if ((v & 1u) == 0)
        return ((uint64_t)out[1] << 32) | out[0];
    return ((uint64_t)out[3] << 32) | out[2];
}

void oracle_vertex_keys(uint64_t seed, uint64_t step, uint64_t N, uint64_t *keys)
{
    for (uint64_t v = 0; v < N; ++v)
        keys[v] = oracle_vertex_key(seed, step, v);
}

/* ------------------------------------------------------------------------------------------ */
/* Eq. 20: uniform B-subset, returned ascending                                                 */
/* ------------------------------------------------------------------------------------------ */

typedef struct { uint64_t key; uint64_t v; } keyed_vertex;

static int cmp_keyed(const void *a, const void *b)
{
    const keyed_vertex *x = (const keyed_vertex *)a, *y = (const keyed_vertex *)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->v != y->v) return x->v < y->v ? -1 : 1;
    return 0;
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Returns 0, or -1 on invalid arguments / allocation failure. */
int oracle_sample_uniform(uint64_t N, uint64_t B, uint64_t seed, uint64_t step, int32_t *S)
{
    if (B == 0 || B > N || N > 0x7fffffffull) return -1;
    keyed_vertex *all = (keyed_vertex *)malloc(sizeof(keyed_vertex) * N);
    if (!all) return -1;
    for (uint64_t v = 0; v < N; ++v) {
        all[v].key = oracle_vertex_key(seed, step, v);
        all[v].v = v;
    }
    qsort(all, N, sizeof(keyed_vertex), cmp_keyed);
    for (uint64_t i = 0; i < B; ++i) S[i] = (int32_t)all[i].v;
    free(all);
    qsort(S, B, sizeof(int32_t), cmp_i32);
    return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* Eqs. 21, 23, 24: induced, normalised, rescaled subgraph as CSR                               */
/* ------------------------------------------------------------------------------------------ */

/* index of u in ascending S, or -1 */
static int64_t find_in_sample(const int32_t *S, int64_t B, int32_t u)
{
    int64_t lo = 0, hi = B - 1;
    while (lo <= hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (S[mid] == u) return mid;
        if (S[mid] < u) lo = mid + 1; else hi = mid - 1;
    }
    return -1;
}

/*
 * Input: canonical CSR of A + I on N vertices (ascending unique columns, one self-loop a row).
 *   val == NULL: a_vu = 1 / sqrt(deg(v) deg(u)) with deg = row length (self-loop included), Eq. 3;
 *   val != NULL: a_vu = val[e] verbatim (Algorithm 2 takes the weights as an input).
 * norm_mode 0: weights inherited from the full graph (Sec. III-D, below Eq. 21).
 * norm_mode 1: degrees recounted on the induced subgraph (val is ignored).
 * rescale 1:  off-diagonal entries divided by p = (B-1)/(N-1), Eqs. 23-24; diagonal untouched.
 * Output rows follow ascending S, columns are positions in S, ascending within a row.
 * Returns nnz (entries beyond `capacity` are counted but not written), or -1 on bad arguments.
 */
int64_t oracle_induced_csr(uint64_t N, const int64_t *rowptr, const int32_t *colidx, const float *val,
                           const int32_t *S, uint64_t B, int norm_mode, int rescale,
                           int32_t *rowptr_S, int32_t *colidx_S, float *val_S, int64_t capacity)
{
    if (B == 0 || B > N) return -1;
    /* p = Pr[u in S | v in S], Eq. 23.  With B == 1 no off-diagonal entry survives, p is unused. */
    double p = 1.0;
    if (rescale && B > 1) p = ((double)B - 1.0) / ((double)N - 1.0);
    int64_t nnz = 0;
    rowptr_S[0] = 0;
    for (uint64_t i = 0; i < B; ++i) {
        int64_t v = S[i];
        double deg_v = (double)(rowptr[v + 1] - rowptr[v]);
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            int32_t u = colidx[e];
            int64_t j = find_in_sample(S, (int64_t)B, u);
            if (j < 0) continue;
            if (nnz < capacity) {
                double a;
                if (val) a = (double)val[e];
                else {
                    double deg_u = (double)(rowptr[(int64_t)u + 1] - rowptr[u]);
                    a = 1.0 / sqrt(deg_v * deg_u);
                }
                if (u != v) a /= p;
                colidx_S[nnz] = (int32_t)j;
                val_S[nnz] = (float)a;
            }
            ++nnz;
        }
        rowptr_S[i + 1] = (int32_t)nnz;
    }
    if (norm_mode == 1) {
        int64_t lim = nnz < capacity ? nnz : capacity;
        for (uint64_t i = 0; i < B; ++i) {
            double di = (double)(rowptr_S[i + 1] - rowptr_S[i]);
            for (int64_t e = rowptr_S[i]; e < rowptr_S[i + 1] && e < lim; ++e) {
                int32_t j = colidx_S[e];
                double dj = (double)(rowptr_S[j + 1] - rowptr_S[j]);
                double a = 1.0 / sqrt(di * dj);
                if ((uint64_t)j != i) a /= p;
                val_S[e] = (float)a;
            }
        }
    }
    return nnz;
}

/*
 * One shard of the same matrix (Algorithm 2 with a row range [R0, R1) and a column range [C0, C1) of
 * global vertex ids): the B x B matrix restricted to the rows of S inside the row range (S_r, Alg. 2
 * line 4) and the columns of S inside the column range (S_c, line 5), in the same [0, B) namespace;
 * rows outside the row range are empty.  Weights as in norm_mode 0 (full-graph degrees, or val).
 */
int64_t oracle_induced_csr_range(uint64_t N, const int64_t *rowptr, const int32_t *colidx, const float *val,
                                 const int32_t *S, uint64_t B, int rescale, int64_t R0, int64_t R1, int64_t C0,
                                 int64_t C1, int32_t *rowptr_S, int32_t *colidx_S, float *val_S, int64_t capacity)
{
    if (B == 0 || B > N) return -1;
    if (R0 < 0 || R1 < R0 || (uint64_t)R1 > N || C0 < 0 || C1 < C0 || (uint64_t)C1 > N) return -1;
    double p = 1.0;
    if (rescale && B > 1) p = ((double)B - 1.0) / ((double)N - 1.0);
    int64_t nnz = 0;
    rowptr_S[0] = 0;
    for (uint64_t i = 0; i < B; ++i) {
        int64_t v = S[i];
        if (v >= R0 && v < R1) {
            double deg_v = (double)(rowptr[v + 1] - rowptr[v]);
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                int32_t u = colidx[e];
                if (u < C0 || u >= C1) continue;
                int64_t j = find_in_sample(S, (int64_t)B, u);
                if (j < 0) continue;
                if (nnz < capacity) {
                    double a;
                    if (val) a = (double)val[e];
                    else {
                        double deg_u = (double)(rowptr[(int64_t)u + 1] - rowptr[u]);
                        a = 1.0 / sqrt(deg_v * deg_u);
                    }
                    if (u != v) a /= p;
                    colidx_S[nnz] = (int32_t)j;
                    val_S[nnz] = (float)a;
                }
                ++nnz;
            }
        }
        rowptr_S[i + 1] = (int32_t)nnz;
    }
    return nnz;
}

/* ------------------------------------------------------------------------------------------ */
/* Eq. 26: slicing                                                                              */
/* ------------------------------------------------------------------------------------------ */

void oracle_gather_rows(const float *X, int64_t d, const int32_t *S, int64_t B, double *out)
{
    for (int64_t i = 0; i < B; ++i)
        for (int64_t j = 0; j < d; ++j)
            out[i * d + j] = (double)X[(int64_t)S[i] * d + j];
}

void oracle_gather_labels(const int32_t *Y, const int32_t *S, int64_t B, int32_t *out)
{
    for (int64_t i = 0; i < B; ++i) out[i] = Y[S[i]];
}

/* ------------------------------------------------------------------------------------------ */
/* Eqs. 5-6 and the layer                                                                       */
/* ------------------------------------------------------------------------------------------ */

/* bfloat16 rounding (round to nearest, ties to even) of a double that already holds an fp32-
 * representable or wider value: first to fp32, then the top 16 bits of that. */
double oracle_round_bf16(double x)
{
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return (double)f; /* inf / nan unchanged */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* the same rounding, element by element, over an array (dst may be src) */
void oracle_round_bf16_array(const double *src, double *dst, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = oracle_round_bf16(src[i]);
}

/* out[i,:] = sum_e val[e] * H[col[e],:]  (Eq. 5) */
void oracle_spmm(int64_t rows, const int32_t *rowptr, const int32_t *colidx, const float *val,
                 const double *H, int64_t d, double *out)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < rows; ++i) {
        double *o = out + i * d;
        for (int64_t j = 0; j < d; ++j) o[j] = 0.0;
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            double a = (double)val[e];
            const double *h = H + (int64_t)colidx[e] * d;
            for (int64_t j = 0; j < d; ++j) o[j] += a * h[j];
        }
    }
}

/* Explicit transpose of a CSR with `rows` rows and `cols` columns (counting sort on columns). */
void oracle_csr_transpose(int64_t rows, int64_t cols, const int32_t *rowptr, const int32_t *colidx,
                          const float *val, int32_t *rowptr_T, int32_t *colidx_T, float *val_T)
{
    for (int64_t j = 0; j <= cols; ++j) rowptr_T[j] = 0;
    for (int64_t e = 0; e < rowptr[rows]; ++e) rowptr_T[colidx[e] + 1]++;
    for (int64_t j = 0; j < cols; ++j) rowptr_T[j + 1] += rowptr_T[j];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(cols > 0 ? cols : 1));
    for (int64_t j = 0; j < cols; ++j) cursor[j] = rowptr_T[j];
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            int32_t q = cursor[colidx[e]]++;
            colidx_T[q] = (int32_t)i;
            val_T[q] = val[e];
        }
    free(cursor);
}

/* C[M x N] = A[M x K] * B[K x N], row-major, plain triple loop (Eq. 6) */
void oracle_gemm(int64_t M, int64_t K, int64_t N, const double *A, const double *B, double *C)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *c = C + i * N;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double a = A[i * K + k];
            const double *b = B + k * N;
            for (int64_t j = 0; j < N; ++j) c[j] += a * b[j];
        }
    }
}

static void round_copy(const double *src, double *dst, int64_t n, int bf16)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = bf16 ? oracle_round_bf16(src[i]) : src[i];
}

/*
 * One GCN layer forward: T = A_S H (Eq. 5), Z = T W + b (Eq. 6; the bias is an extension, NULL
 * for none), Y = max(Z, 0) when relu (Eq. 8) else Z.  With bf16 != 0 the two GEMM operands T and W
 * are rounded to bfloat16 before the product (accumulation stays in double); T is returned
 * unrounded.
 */
void oracle_gcn_fwd(int64_t B, const int32_t *rowptr, const int32_t *colidx, const float *val,
                    const double *H, int64_t d_in, const double *W, int64_t d_out, const double *bias,
                    int relu, int bf16, double *T, double *Y)
{
    oracle_spmm(B, rowptr, colidx, val, H, d_in, T);
    double *Tr = T, *Wr = (double *)W;
    if (bf16) {
        Tr = (double *)malloc(sizeof(double) * (size_t)(B * d_in));
        Wr = (double *)malloc(sizeof(double) * (size_t)(d_in * d_out));
        round_copy(T, Tr, B * d_in, 1);
        round_copy(W, Wr, d_in * d_out, 1);
    }
    oracle_gemm(B, d_in, d_out, Tr, Wr, Y);
    if (bf16) { free(Tr); free(Wr); }
    for (int64_t i = 0; i < B; ++i)
        for (int64_t j = 0; j < d_out; ++j) {
            double z = Y[i * d_out + j] + (bias ? bias[j] : 0.0);
            if (relu && !(z > 0.0)) z = 0.0;
            Y[i * d_out + j] = z;
        }
}

/*
 * Layer backward (Sec. III-C).  dZ = dY where Y > 0 (all of dY when relu == 0); db = column sums of
 * dZ; dW = T^T dZ; dT = dZ W^T; dH = A_S^T dT, computed with the explicitly transposed CSR
 * (rowptr_T, colidx_T, val_T).  dH may be NULL (first layer: features are not trained).  With
 * bit 0 of bf16 set the operands of both GEMMs (T, dZ, W) are rounded to bfloat16 first; with bit 1
 * set the gradient of the aggregate, dT = dZ W^T, is stored as bfloat16 (rounded once) before the
 * transposed sparse product reads it.
 */
void oracle_gcn_bwd(int64_t B, const int32_t *rowptr_T, const int32_t *colidx_T, const float *val_T,
                    const double *T, int64_t d_in, const double *W, int64_t d_out, const double *Y,
                    const double *dY, int relu, int bf16, double *dH, double *dW, double *db)
{
    double *dZ = (double *)malloc(sizeof(double) * (size_t)(B * d_out));
    for (int64_t i = 0; i < B * d_out; ++i)
        dZ[i] = (!relu || Y[i] > 0.0) ? dY[i] : 0.0;
    if (db) {
        for (int64_t j = 0; j < d_out; ++j) db[j] = 0.0;
        for (int64_t i = 0; i < B; ++i)
            for (int64_t j = 0; j < d_out; ++j) db[j] += dZ[i * d_out + j];
    }
    double *Tr = (double *)malloc(sizeof(double) * (size_t)(B * d_in));
    double *Wr = (double *)malloc(sizeof(double) * (size_t)(d_in * d_out));
    const int round_operands = bf16 & 1, store_dT_bf16 = bf16 & 2;
    round_copy(T, Tr, B * d_in, round_operands);
    round_copy(W, Wr, d_in * d_out, round_operands);
    if (round_operands) round_copy(dZ, dZ, B * d_out, 1);
    /* dW[k, j] = sum_i T[i, k] dZ[i, j] */
    for (int64_t k = 0; k < d_in * d_out; ++k) dW[k] = 0.0;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < d_in; ++k)
        for (int64_t i = 0; i < B; ++i) {
            double t = Tr[i * d_in + k];
            for (int64_t j = 0; j < d_out; ++j) dW[k * d_out + j] += t * dZ[i * d_out + j];
        }
    if (dH) {
        double *dT = (double *)malloc(sizeof(double) * (size_t)(B * d_in));
        /* dT[i, k] = sum_j dZ[i, j] W[k, j] */
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < B; ++i)
            for (int64_t k = 0; k < d_in; ++k) {
                double s = 0.0;
                for (int64_t j = 0; j < d_out; ++j) s += dZ[i * d_out + j] * Wr[k * d_out + j];
                dT[i * d_in + k] = s;
            }
        if (store_dT_bf16) round_copy(dT, dT, B * d_in, 1);
        oracle_spmm(B, rowptr_T, colidx_T, val_T, dT, d_in, dH);
        free(dT);
    }
    free(Tr); free(Wr); free(dZ);
}

/* Mean softmax cross-entropy over B rows and its gradient dO = (softmax(O) - onehot(y)) / B. */
double oracle_softmax_xent(int64_t B, int64_t C, const double *O, const int32_t *labels, double *dO)
{
    double loss = 0.0;
    for (int64_t i = 0; i < B; ++i) {
        const double *o = O + i * C;
        double m = o[0];
        for (int64_t j = 1; j < C; ++j) if (o[j] > m) m = o[j];
        double s = 0.0;
        for (int64_t j = 0; j < C; ++j) s += exp(o[j] - m);
        double lse = m + log(s);
        loss += lse - o[labels[i]];
        if (dO)
            for (int64_t j = 0; j < C; ++j)
                dO[i * C + j] = (exp(o[j] - lse) - (j == labels[i] ? 1.0 : 0.0)) / (double)B;
    }
    return loss / (double)B;
}

/* ------------------------------------------------------------------------------------------ */
/* Layer tail (Eqs. 7-10): Y = dropout(relu(rmsnorm(Z))) + R                                    */

/* 1 if element e of layer `layer` at step `step` survives dropout with drop probability q. */
int oracle_dropout_keep(uint64_t seed, uint32_t layer, uint64_t step, uint64_t e, double q)
{
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    const uint64_t blk = e / 4;
    const uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)step, 0x80000000u + layer};
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    const uint32_t thr = (uint32_t)floor(q * 4294967296.0);
    return out[e % 4] >= thr;
}

void oracle_dropout_mask(uint64_t seed, uint32_t layer, uint64_t step, uint64_t n, double q, uint8_t *keep)
{
    for (uint64_t e = 0; e < n; ++e) keep[e] = (uint8_t)oracle_dropout_keep(seed, layer, step, e, q);
}

/*
 * Forward.  Z: B x d (the convolution output X_conv), gamma: d (NULL = ones), R: B x d residual
 * input X_{h,l-1} or NULL.  Y: B x d out.  Optional outputs (NULL to skip): inv_rms[B] =
 * 1 / sqrt(mean(z^2) + eps), Xn: B x d the normalised values of Eq. 7.
 */
void oracle_tail_fwd(int64_t B, int64_t d, const double *Z, const double *gamma, double eps, const double *R,
                     double q, uint64_t seed, uint32_t layer, uint64_t step, double *Y, double *inv_rms, double *Xn)
{
    const double scale = q > 0.0 ? 1.0 / (1.0 - q) : 1.0;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < B; ++i) {
        double ss = 0.0;
        for (int64_t j = 0; j < d; ++j) ss += Z[i * d + j] * Z[i * d + j];
        const double ir = 1.0 / sqrt(ss / (double)d + eps);                           /* Eq. 7 */
        if (inv_rms) inv_rms[i] = ir;
        for (int64_t j = 0; j < d; ++j) {
            const double n = (gamma ? gamma[j] : 1.0) * Z[i * d + j] * ir;
            if (Xn) Xn[i * d + j] = n;
            double r = n > 0.0 ? n : 0.0;                                             /* Eq. 8 */
            if (q > 0.0) r = oracle_dropout_keep(seed, layer, step, (uint64_t)(i * d + j), q) ? r * scale : 0.0; /* Eq. 9 */
            Y[i * d + j] = r + (R ? R[i * d + j] : 0.0);                              /* Eq. 10 */
        }
    }
}

/*
 * Backward of the main branch (Sec. III-C: dropout mask, ReLU mask, RMSNorm backward): given
 * dY = grad of Y, returns dZ (B x d) and dgamma (d, NULL to skip).  The gradient of the skip path
 * is dY itself (Eq. 10) and is not formed here.
 * With zhat = z * inv_rms and n = gamma * zhat:  dn = dY * M_drop * [n > 0],
 * dgamma = sum_i dn * zhat,  dzhat = dn * gamma,  dz = (dzhat - zhat * mean_j(dzhat * zhat)) * inv_rms.
 */
void oracle_tail_bwd(int64_t B, int64_t d, const double *Z, const double *gamma, double eps, double q, uint64_t seed,
                     uint32_t layer, uint64_t step, const double *dY, double *dZ, double *dgamma)
{
    const double scale = q > 0.0 ? 1.0 / (1.0 - q) : 1.0;
    if (dgamma) for (int64_t j = 0; j < d; ++j) dgamma[j] = 0.0;
    double *dn = (double *)malloc(sizeof(double) * (size_t)(d > 0 ? d : 1));
    for (int64_t i = 0; i < B; ++i) {
        double ss = 0.0;
        for (int64_t j = 0; j < d; ++j) ss += Z[i * d + j] * Z[i * d + j];
        const double ir = 1.0 / sqrt(ss / (double)d + eps);
        double dot = 0.0;
        for (int64_t j = 0; j < d; ++j) {
            const double g = gamma ? gamma[j] : 1.0, zh = Z[i * d + j] * ir, n = g * zh;
            double m = n > 0.0 ? 1.0 : 0.0;
            if (q > 0.0) m *= oracle_dropout_keep(seed, layer, step, (uint64_t)(i * d + j), q) ? scale : 0.0;
            dn[j] = dY[i * d + j] * m;
            if (dgamma) dgamma[j] += dn[j] * zh;
            dot += dn[j] * g * zh;
        }
        dot /= (double)d;
        for (int64_t j = 0; j < d; ++j) {
            const double g = gamma ? gamma[j] : 1.0, zh = Z[i * d + j] * ir;
            dZ[i * d + j] = (dn[j] * g - zh * dot) * ir;
        }
    }
    free(dn);
}

/*
 * Binary cross-entropy on logits, the paper's loss for multi-label tasks (Sec. III-B "Output Head and
 * Loss"): mean over the B x C entries of  -[y log s(o) + (1 - y) log(1 - s(o))],  s = logistic function,
 * written as max(o, 0) - o y + log(1 + exp(-|o|)); dO = (s(o) - y) / (B C).  Y holds the targets (0 / 1,
 * any value in [0, 1] is accepted).  The paper does not say mean or sum: the mean is the reading taken.
 */
double oracle_sigmoid_bce(int64_t B, int64_t C, const double *O, const double *Y, double *dO)
{
    double loss = 0.0;
    const double inv = 1.0 / ((double)B * (double)C);
    for (int64_t i = 0; i < B * C; ++i) {
        const double o = O[i], y = Y[i];
        loss += (o > 0.0 ? o : 0.0) - o * y + log1p(exp(-fabs(o)));
        const double sg = o >= 0.0 ? 1.0 / (1.0 + exp(-o)) : exp(o) / (1.0 + exp(o));
        if (dO) dO[i] = (sg - y) * inv;
    }
    return loss * inv;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
