/*
 * fp64 CPU oracle that never forms an S x S matrix.  TEST INFRASTRUCTURE ONLY.
 *
 * Same operator as oracle/ref_numpy.py, organised so that large sequences and
 * sampled rows / columns are affordable:
 *   - a ROW pass computes, for each requested query row i and each query head,
 *     the scores against the visible keys, LSE_i, O_i and (when dO is given)
 *     Delta_i and dQ_i;
 *   - a COLUMN pass computes dK_j and dV_j of requested key positions j as the
 *     sums over the participating query rows i >= j, re-evaluating s_ij from
 *     q_i and k_j and using LSE_i / Delta_i from the row pass.
 * Both follow the definition term by term:
 *     s_ij = scale * q_i . k_j             (j <= i, same document)
 *     LSE_i = log sum_j exp(s_ij),  P_ij = exp(s_ij - LSE_i),  O_i = sum_j P_ij v_j
 *     Delta_i = dO_i . O_i,  dP_ij = dO_i . v_j,  dS_ij = P_ij (dP_ij - Delta_i)
 *     dQ_i = scale sum_j dS_ij k_j
 *     dK_j = scale sum_{a in group} sum_i dS_ij q_i,   dV_j = sum_{a in group} sum_i P_ij dO_i
 * Query head a uses key/value head a / G, G = Hq / Hkv (grouped-query or full
 * attention; paper Section 4 setup).  Attention runs over the full sequence
 * for this device's heads (Section 2, Figure 1).  Documents given by
 * cu_seqlens are independent (block-diagonal causal); one document [0,T) is
 * the dense causal case.
 *
 * Tensors are row-major [T, H, D] doubles.  No blocking, no fusion beyond the
 * two passes; the only liberty is that a dot product keeps four partial sums.
 * It includes nothing from, and links nothing of, the HIP library.
 *
 * Pinned by tests/test_oracle_pins.py against brute force, closed forms and
 * the dense numpy writing of the same definition.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int ref_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- re-layout: out[b, p*S_l + s, j, :] = in[b, s, p*h + j, :] ------------ */
void ref_pack_seq_to_head(const void* in, void* out, int64_t B, int64_t S_l, int64_t H,
                          int64_t D, int32_t P, int32_t elem_bytes) {
    const char* src = (const char*)in;
    char* dst = (char*)out;
    const int64_t h = H / P;
    const int64_t vec = D * elem_bytes;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t s = 0; s < S_l; ++s)
                for (int64_t j = 0; j < h; ++j)
                    memcpy(dst + (((b * P * S_l) + p * S_l + s) * h + j) * vec,
                           src + (((b * S_l) + s) * H + p * h + j) * vec, (size_t)vec);
}

/* ---- inverse: out[b, s, p*h + j, :] = in[b, p*S_l + s, j, :] -------------- */
void ref_unpack_head_to_seq(const void* in, void* out, int64_t B, int64_t S_l, int64_t H,
                            int64_t D, int32_t P, int32_t elem_bytes) {
    const char* src = (const char*)in;
    char* dst = (char*)out;
    const int64_t h = H / P;
    const int64_t vec = D * elem_bytes;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t s = 0; s < S_l; ++s)
                for (int64_t j = 0; j < h; ++j)
                    memcpy(dst + (((b * S_l) + s) * H + p * h + j) * vec,
                           src + (((b * P * S_l) + p * S_l + s) * h + j) * vec, (size_t)vec);
}

static double dot(const double* a, const double* b, int D) {
    double s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    int d = 0;
    for (; d + 4 <= D; d += 4) {
        s0 += a[d] * b[d];
        s1 += a[d + 1] * b[d + 1];
        s2 += a[d + 2] * b[d + 2];
        s3 += a[d + 3] * b[d + 3];
    }
    for (; d < D; ++d) s0 += a[d] * b[d];
    return (s0 + s1) + (s2 + s3);
}

/* first row of the document that contains row i (cu is non-decreasing, cu[0]=0) */
static int64_t doc_start(const int32_t* cu, int n_docs, int64_t i) {
    int64_t start = 0;
    for (int t = 0; t < n_docs; ++t)
        if ((int64_t)cu[t] <= i && i < (int64_t)cu[t + 1]) start = cu[t];
    return start;
}

static int64_t doc_end(const int32_t* cu, int n_docs, int64_t i) {
    int64_t end = 0;
    for (int t = 0; t < n_docs; ++t)
        if ((int64_t)cu[t] <= i && i < (int64_t)cu[t + 1]) end = cu[t + 1];
    return end;
}

/*
 * ROW pass.  rows[n_rows] are global positions.  Outputs (any may be NULL):
 *   O_rows [n_rows, Hq, D], lse_rows [Hq, n_rows],
 *   delta_rows [Hq, n_rows], dQ_rows [n_rows, Hq, D]   (the last two need dO).
 * Returns 0, or -1 on allocation failure.
 */
int ref_attn_rows(const double* q, const double* k, const double* v, const double* dO,
                  const int32_t* cu, int32_t n_docs, int64_t T, int32_t Hq, int32_t Hkv,
                  int32_t D, double scale, const int64_t* rows, int64_t n_rows,
                  double* O_rows, double* lse_rows, double* delta_rows, double* dQ_rows) {
    const int G = Hq / Hkv;
    int fail = 0;
    (void)T;
#pragma omp parallel
    {
        double* s = NULL;
        int64_t cap = 0;
        double* o = (double*)malloc(sizeof(double) * (size_t)D);
        double* dq = (double*)malloc(sizeof(double) * (size_t)D);
        if (!o || !dq) fail = 1;
#pragma omp for schedule(dynamic, 1) collapse(2)
        for (int64_t r = 0; r < n_rows; ++r) {
            for (int a = 0; a < Hq; ++a) {
                if (fail) continue;
                const int64_t i = rows[r];
                const int g = a / G;
                const int64_t j0 = doc_start(cu, n_docs, i);
                const int64_t n = i - j0 + 1; /* visible keys j0..i */
                if (n > cap) {
                    free(s);
                    cap = n;
                    s = (double*)malloc(sizeof(double) * (size_t)cap);
                    if (!s) { fail = 1; cap = 0; continue; }
                }
                const double* qi = q + ((size_t)i * Hq + a) * D;
                double m = -INFINITY;
                for (int64_t j = 0; j < n; ++j) {
                    s[j] = scale * dot(qi, k + ((size_t)(j0 + j) * Hkv + g) * D, D);
                    if (s[j] > m) m = s[j];
                }
                double sum = 0;
                for (int64_t j = 0; j < n; ++j) sum += exp(s[j] - m);
                const double lse = m + log(sum);
                for (int d = 0; d < D; ++d) o[d] = 0;
                for (int64_t j = 0; j < n; ++j) {
                    const double p = exp(s[j] - lse);
                    const double* vj = v + ((size_t)(j0 + j) * Hkv + g) * D;
                    for (int d = 0; d < D; ++d) o[d] += p * vj[d];
                    s[j] = p; /* keep P_ij for the gradient below */
                }
                if (O_rows) memcpy(O_rows + ((size_t)r * Hq + a) * D, o, sizeof(double) * (size_t)D);
                if (lse_rows) lse_rows[(size_t)a * n_rows + r] = lse;
                if (dO && (delta_rows || dQ_rows)) {
                    const double* doi = dO + ((size_t)i * Hq + a) * D;
                    const double delta = dot(doi, o, D);
                    if (delta_rows) delta_rows[(size_t)a * n_rows + r] = delta;
                    if (dQ_rows) {
                        for (int d = 0; d < D; ++d) dq[d] = 0;
                        for (int64_t j = 0; j < n; ++j) {
                            const double dp = dot(doi, v + ((size_t)(j0 + j) * Hkv + g) * D, D);
                            const double ds = s[j] * (dp - delta);
                            const double* kj = k + ((size_t)(j0 + j) * Hkv + g) * D;
                            for (int d = 0; d < D; ++d) dq[d] += ds * kj[d];
                        }
                        double* out = dQ_rows + ((size_t)r * Hq + a) * D;
                        for (int d = 0; d < D; ++d) out[d] = scale * dq[d];
                    }
                }
            }
        }
        free(s);
        free(o);
        free(dq);
    }
    return fail ? -1 : 0;
}

/*
 * COLUMN pass.  rows[n_rows] (ascending) are the query rows that take part
 * (all rows for the full gradient; the rows where dO is non-zero otherwise),
 * with their lse_rows / delta_rows [Hq, n_rows] from the row pass.
 * cols[n_cols] are the key positions wanted.  Outputs dK_cols, dV_cols
 * [n_cols, Hkv, D].
 */
int ref_attn_cols(const double* q, const double* k, const double* v, const double* dO,
                  const int32_t* cu, int32_t n_docs, int64_t T, int32_t Hq, int32_t Hkv,
                  int32_t D, double scale, const int64_t* rows, int64_t n_rows,
                  const double* lse_rows, const double* delta_rows, const int64_t* cols,
                  int64_t n_cols, double* dK_cols, double* dV_cols) {
    const int G = Hq / Hkv;
    (void)T;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int64_t c = 0; c < n_cols; ++c) {
        for (int g = 0; g < Hkv; ++g) {
            const int64_t j = cols[c];
            const int64_t jend = doc_end(cu, n_docs, j); /* rows j..jend-1 see key j */
            const double* kj = k + ((size_t)j * Hkv + g) * D;
            const double* vj = v + ((size_t)j * Hkv + g) * D;
            double* dk = dK_cols + ((size_t)c * Hkv + g) * D;
            double* dv = dV_cols + ((size_t)c * Hkv + g) * D;
            for (int d = 0; d < D; ++d) { dk[d] = 0; dv[d] = 0; }
            for (int a = g * G; a < (g + 1) * G; ++a) {
                for (int64_t r = 0; r < n_rows; ++r) {
                    const int64_t i = rows[r];
                    if (i < j || i >= jend) continue;
                    const double* qi = q + ((size_t)i * Hq + a) * D;
                    const double* doi = dO + ((size_t)i * Hq + a) * D;
                    const double p = exp(scale * dot(qi, kj, D) - lse_rows[(size_t)a * n_rows + r]);
                    const double dp = dot(doi, vj, D);
                    const double ds = p * (dp - delta_rows[(size_t)a * n_rows + r]);
                    for (int d = 0; d < D; ++d) {
                        dv[d] += p * doi[d];
                        dk[d] += ds * qi[d];
                    }
                }
            }
            for (int d = 0; d < D; ++d) dk[d] *= scale;
        }
    }
    return 0;
}
