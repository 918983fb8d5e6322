/*
 * CPU oracle for the CSR SpMM / SDDMM / row-softmax / CSR-attention hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP sources, and nothing in the product path may call it: only the
 * tests, the smoke check and the benchmark's CPU-baseline leg do.
 *
 * Everything is accumulated in double precision.  Inputs are fp32 (dtype 0) or
 * bf16 bit patterns (dtype 1); both convert to double exactly.  Rows are
 * independent, so the outer loop over rows may run under OpenMP without
 * changing any sum: each output element is produced by one thread, in CSR
 * storage order.
 *
 * What each function follows:
 *   oracle_spmm          Notation paragraph: C = A B, A sparse CSR, B dense.
 *   oracle_sddmm         Notation paragraph: A~_ij = <X_i, Y_j> on the pattern of A.
 *   oracle_row_softmax   Method / Kernel templates: numerically stable CSR row-softmax.
 *   oracle_csr_attention Preliminaries: SDDMM -> row-softmax -> SpMM.
 *   oracle_hub_partition Kernel-variant table: heavy rows (degree >= hubT) vs others;
 *                        the chunking of heavy rows is this project's own scheme.
 *   oracle_decide        Scheduler subsection + decision sketch + Proposition 1.
 *   oracle_csr_transpose, oracle_row_softmax_backward, oracle_csr_attention_backward
 *                        the adjoints needed when the operators sit in a training step (Introduction:
 *                        training throughput is bounded by these aggregations): d/dB of C = A B is A^T dC,
 *                        the Jacobian-transpose product of the row-softmax, and the chain rule through the
 *                        three steps of the attention pipeline.
 *
 * All pins for these functions live in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F32 0
#define ORACLE_BF16 1

static double load_as_double(const void* base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32) {
        return (double)((const float*)base)[idx];
    } else {
        uint32_t bits = ((uint32_t)((const uint16_t*)base)[idx]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* C[i,f] = sum over stored p of row i of val[p] * B[colind[p], f].  Empty row -> zeros. */
int oracle_spmm(int64_t n_rows, const int32_t* rowptr, const int32_t* colind, const float* val,
                const void* B, int64_t ldb, int32_t F, int dtype, double* C, int64_t ldc)
{
    int64_t i;
#pragma omp parallel for schedule(dynamic, 256)
    for (i = 0; i < n_rows; ++i) {
        for (int32_t f = 0; f < F; ++f) {
            double acc = 0.0;
            for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
                acc += (double)val[p] * load_as_double(B, (int64_t)colind[p] * ldb + f, dtype);
            }
            C[i * ldc + f] = acc;
        }
    }
    return 0;
}

/* out[p] = sum_f X[i,f] * Y[colind[p], f] for every stored p of row i; val is not used. */
int oracle_sddmm(int64_t n_rows, const int32_t* rowptr, const int32_t* colind,
                 const void* X, int64_t ldx, const void* Y, int64_t ldy, int32_t F, int dtype,
                 double* out)
{
    int64_t i;
#pragma omp parallel for schedule(dynamic, 256)
    for (i = 0; i < n_rows; ++i) {
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            double acc = 0.0;
            for (int32_t f = 0; f < F; ++f) {
                acc += load_as_double(X, i * ldx + f, dtype) *
                       load_as_double(Y, (int64_t)colind[p] * ldy + f, dtype);
            }
            out[p] = acc;
        }
    }
    return 0;
}

/* s and out are [nnz, H] (head minor).  For every row i and head h with deg(i) > 0:
 * m = max_p s[p,h]; e_p = exp(s[p,h] - m); out[p,h] = e_p / sum_q e_q.  Empty rows write nothing. */
int oracle_row_softmax(int64_t n_rows, const int32_t* rowptr, const double* s, int32_t H, double* out)
{
    int64_t i;
#pragma omp parallel for schedule(dynamic, 256)
    for (i = 0; i < n_rows; ++i) {
        int64_t p0 = rowptr[i], p1 = rowptr[i + 1];
        if (p1 <= p0) continue;
        for (int32_t h = 0; h < H; ++h) {
            double m = s[p0 * H + h];
            for (int64_t p = p0 + 1; p < p1; ++p) {
                if (s[p * H + h] > m) m = s[p * H + h];
            }
            double denom = 0.0;
            for (int64_t p = p0; p < p1; ++p) denom += exp(s[p * H + h] - m);
            for (int64_t p = p0; p < p1; ++p) out[p * H + h] = exp(s[p * H + h] - m) / denom;
        }
    }
    return 0;
}

/* Q, K, V are [N, H, d] (d minor).  S[p,h] = scale * <Q[i,h,:], K[j,h,:]>, P = row-softmax(S) per
 * (row, head), O[i,h,:] = sum_p P[p,h] * V[colind[p],h,:].  Rows without nonzeros give O = 0.
 * S_out and P_out ([nnz,H]) may be NULL; O is [N, H, d] doubles. */
int oracle_csr_attention(int64_t N, const int32_t* rowptr, const int32_t* colind,
                         const void* Q, const void* K, const void* V, int32_t H, int32_t d,
                         double scale, int dtype, double* S_out, double* P_out, double* O)
{
    int64_t nnz = rowptr[N];
    double* S = S_out ? S_out : (double*)malloc(sizeof(double) * (size_t)(nnz > 0 ? nnz : 1) * H);
    double* P = P_out ? P_out : (double*)malloc(sizeof(double) * (size_t)(nnz > 0 ? nnz : 1) * H);
    if (!S || !P) return 1;
    int64_t i;
    /* step 1: SDDMM per head, scaled */
#pragma omp parallel for schedule(dynamic, 256)
    for (i = 0; i < N; ++i) {
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int64_t j = colind[p];
            for (int32_t h = 0; h < H; ++h) {
                double acc = 0.0;
                for (int32_t k = 0; k < d; ++k) {
                    acc += load_as_double(Q, (i * H + h) * d + k, dtype) *
                           load_as_double(K, (j * H + h) * d + k, dtype);
                }
                S[p * H + h] = scale * acc;
            }
        }
    }
    /* step 2: row-softmax */
    oracle_row_softmax(N, rowptr, S, H, P);
    /* step 3: SpMM per head with P as the values */
#pragma omp parallel for schedule(dynamic, 256)
    for (i = 0; i < N; ++i) {
        for (int32_t h = 0; h < H; ++h) {
            for (int32_t k = 0; k < d; ++k) {
                double acc = 0.0;
                for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
                    acc += P[p * H + h] * load_as_double(V, ((int64_t)colind[p] * H + h) * d + k, dtype);
                }
                O[(i * H + h) * d + k] = acc;
            }
        }
    }
    if (!S_out) free(S);
    if (!P_out) free(P);
    return 0;
}

/* Heavy/light split and chunking of heavy rows.
 *   hub_rows   : ascending { i : deg(i) >= hub_t }
 *   light_rows : ascending complement (empty rows included)
 *   chunk_ptr  : [n_hub + 1], chunk_ptr[0] = 0, chunk_ptr[k+1] = chunk_ptr[k] + ceil(deg(hub_rows[k]) / hub_chunk)
 * Chunk t of hub row r covers nonzeros [rowptr[r] + t*hub_chunk, min(rowptr[r] + (t+1)*hub_chunk, rowptr[r+1])).
 * Output arrays must hold n_rows (+1 for chunk_ptr) entries. */
int oracle_hub_partition(int64_t n_rows, const int32_t* rowptr, int32_t hub_t, int32_t hub_chunk,
                         int32_t* n_hub, int32_t* hub_rows, int32_t* chunk_ptr,
                         int32_t* n_light, int32_t* light_rows)
{
    int32_t nh = 0, nl = 0;
    if (hub_t < 1 || hub_chunk < 1) return 1;
    chunk_ptr[0] = 0;
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t deg = (int64_t)rowptr[i + 1] - rowptr[i];
        if (deg >= hub_t) {
            int64_t chunks = deg / hub_chunk + (deg % hub_chunk != 0 ? 1 : 0);
            hub_rows[nh] = (int32_t)i;
            chunk_ptr[nh + 1] = chunk_ptr[nh] + (int32_t)chunks;
            ++nh;
        } else {
            light_rows[nl++] = (int32_t)i;
        }
    }
    *n_hub = nh;
    *n_light = nl;
    return 0;
}

/* hist[0] counts rows of degree 0; hist[b], b >= 1, counts rows with 2^(b-1) <= deg < 2^b. */
int oracle_degree_histogram(int64_t n_rows, const int32_t* rowptr, int64_t hist[33], int64_t* max_deg)
{
    int64_t mx = 0;
    for (int b = 0; b < 33; ++b) hist[b] = 0;
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t deg = (int64_t)rowptr[i + 1] - rowptr[i];
        int b = 0;
        for (int64_t t = deg; t > 0; t >>= 1) ++b;
        hist[b] += 1;
        if (deg > mx) mx = deg;
    }
    *max_deg = mx;
    return 0;
}

static uint64_t fnv1a_i64(uint64_t h, int64_t v)
{
    uint64_t u = (uint64_t)v;
    for (int b = 0; b < 8; ++b) {
        h ^= (u >> (8 * b)) & 0xFFu;
        h *= 1099511628211ULL;
    }
    return h;
}

/* 64-bit FNV-1a over the little-endian int64 sequence
 *   n_rows, n_cols, nnz, max_deg, hist[0..32], rowptr[floor(k * n_rows / 1023)] for k = 0..1023. */
uint64_t oracle_graph_signature(int64_t n_rows, int64_t n_cols, const int32_t* rowptr)
{
    int64_t hist[33], max_deg;
    uint64_t h = 14695981039346656037ULL;
    oracle_degree_histogram(n_rows, rowptr, hist, &max_deg);
    h = fnv1a_i64(h, n_rows);
    h = fnv1a_i64(h, n_cols);
    h = fnv1a_i64(h, (int64_t)rowptr[n_rows]);
    h = fnv1a_i64(h, max_deg);
    for (int b = 0; b < 33; ++b) h = fnv1a_i64(h, hist[b]);
    for (int64_t k = 0; k < 1024; ++k) h = fnv1a_i64(h, (int64_t)rowptr[(k * n_rows) / 1023]);
    return h;
}

/* The decision rule: the best candidate is the first one with the strictly smallest probe time;
 * it is accepted iff t_best <= alpha * t_baseline, else the baseline is kept.
 * Returns the index of the accepted candidate, or -1 for the baseline. */
int oracle_decide(int32_t n_cand, const double* t_cand, double t_baseline, double alpha)
{
    int best = -1;
    double tstar = INFINITY;
    for (int32_t c = 0; c < n_cand; ++c) {
        if (t_cand[c] < tstar) {
            best = c;
            tstar = t_cand[c];
        }
    }
    return (tstar <= alpha * t_baseline) ? best : -1;
}

/* A^T as CSR (n_cols rows).  Stable: inside a row of A^T the entries keep the order of their source
 * rows (ascending row index, and storage order for duplicates).  perm[q] = position in A of entry q
 * of A^T, so t_val[q] = val[perm[q]] and t_colind[q] = row of A that owns perm[q].
 * val / t_val may be NULL. */
int oracle_csr_transpose(int64_t n_rows, int64_t n_cols, const int32_t* rowptr, const int32_t* colind,
                         const float* val, int32_t* t_rowptr, int32_t* t_colind, float* t_val, int32_t* perm)
{
    int64_t nnz = rowptr[n_rows];
    int32_t* next = (int32_t*)calloc((size_t)n_cols + 1, sizeof(int32_t));
    if (!next) return 1;
    for (int64_t c = 0; c <= n_cols; ++c) t_rowptr[c] = 0;
    for (int64_t p = 0; p < nnz; ++p) t_rowptr[colind[p] + 1] += 1;
    for (int64_t c = 0; c < n_cols; ++c) t_rowptr[c + 1] += t_rowptr[c];
    for (int64_t c = 0; c < n_cols; ++c) next[c] = t_rowptr[c];
    for (int64_t i = 0; i < n_rows; ++i) {
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int32_t q = next[colind[p]]++;
            t_colind[q] = (int32_t)i;
            if (val && t_val) t_val[q] = val[p];
            perm[q] = (int32_t)p;
        }
    }
    free(next);
    return 0;
}

/* Jacobian-transpose product of the row-softmax: for every row and head,
 * dS[p,h] = P[p,h] * (dP[p,h] - sum_q P[q,h] * dP[q,h]), q over the stored entries of the row. */
int oracle_row_softmax_backward(int64_t n_rows, const int32_t* rowptr, const double* P, const double* dP, int32_t H,
                                double* dS)
{
    int64_t i;
#pragma omp parallel for schedule(dynamic, 256)
    for (i = 0; i < n_rows; ++i) {
        for (int32_t h = 0; h < H; ++h) {
            double dot = 0.0;
            for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) dot += P[p * H + h] * dP[p * H + h];
            for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) dS[p * H + h] = P[p * H + h] * (dP[p * H + h] - dot);
        }
    }
    return 0;
}

/* Adjoint of oracle_csr_attention: given dO = dL/dO ([N, H, d] doubles) it returns dL/dQ, dL/dK, dL/dV
 * ([N, H, d] doubles) by the chain rule through the three steps, in reverse:
 *   O = P V        ->  dV[j,h,:] += P[p,h] * dO[i,h,:],   dP[p,h] = <dO[i,h,:], V[j,h,:]>
 *   P = softmax(S) ->  dS = oracle_row_softmax_backward(P, dP)
 *   S = scale Q K^T on the pattern
 *                  ->  dQ[i,h,:] += scale * dS[p,h] * K[j,h,:],   dK[j,h,:] += scale * dS[p,h] * Q[i,h,:]
 * for every stored p = (i, j).  The scatter into rows j of dK and dV runs serially in storage order. */
int oracle_csr_attention_backward(int64_t N, const int32_t* rowptr, const int32_t* colind,
                                  const void* Q, const void* K, const void* V, const double* dO,
                                  int32_t H, int32_t d, double scale, int dtype,
                                  double* dQ, double* dK, double* dV)
{
    int64_t nnz = rowptr[N];
    size_t cells = (size_t)(nnz > 0 ? nnz : 1) * H;
    double* P = (double*)malloc(sizeof(double) * cells);
    double* dP = (double*)malloc(sizeof(double) * cells);
    double* dS = (double*)malloc(sizeof(double) * cells);
    double* O = (double*)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1) * H * d);
    if (!P || !dP || !dS || !O) return 1;
    double* S = (double*)malloc(sizeof(double) * cells);
    if (!S) return 1;
    oracle_csr_attention(N, rowptr, colind, Q, K, V, H, d, scale, dtype, S, P, O);
    for (int64_t e = 0; e < N * H * d; ++e) dQ[e] = dK[e] = dV[e] = 0.0;
    for (int64_t i = 0; i < N; ++i) {
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int64_t j = colind[p];
            for (int32_t h = 0; h < H; ++h) {
                double acc = 0.0;
                for (int32_t k = 0; k < d; ++k) {
                    double g = dO[(i * H + h) * d + k];
                    acc += g * load_as_double(V, (j * H + h) * d + k, dtype);
                    dV[(j * H + h) * d + k] += P[p * H + h] * g;
                }
                dP[p * H + h] = acc;
            }
        }
    }
    oracle_row_softmax_backward(N, rowptr, P, dP, H, dS);
    for (int64_t i = 0; i < N; ++i) {
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int64_t j = colind[p];
            for (int32_t h = 0; h < H; ++h) {
                double w = scale * dS[p * H + h];
                for (int32_t k = 0; k < d; ++k) {
                    dQ[(i * H + h) * d + k] += w * load_as_double(K, (j * H + h) * d + k, dtype);
                    dK[(j * H + h) * d + k] += w * load_as_double(Q, (i * H + h) * d + k, dtype);
                }
            }
        }
    }
    free(S);
    free(P);
    free(dP);
    free(dS);
    free(O);
    return 0;
}
