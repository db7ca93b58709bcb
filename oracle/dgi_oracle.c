/*
 * dgi_oracle.c — CPU oracle for layer-wise GNN inference.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the reference the GPU library is checked against.  It is deliberately plain and slow:
 * one loop nest per definition, double accumulation, no blocking, no transform-before-aggregate
 * trick, no batching, no reordering.  It shares no code with the GPU library and is never called
 * by it: only tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * What it computes (DGI paper, arXiv 2211.15082):
 *   - Eq. 1 (Section 1): h^l_v = AGGREGATE^l({h^{l-1}_u : u in N(v)} ∪ v ; w^l), N(v) = in-neighbours,
 *     instantiated with the textbook layers named in Section 5 (GCN, GAT) and GraphSAGE-mean:
 *       SUM / MEAN : h'_v = act(h_v W_self + m_v W_neigh + b),  m_v = sum or mean of h_u over N(v)
 *       GCN        : h'_v = act((sum_u h_u / sqrt(d_out(u) d_in(v))) W + b)
 *       GAT        : z_u = h_u W as [heads, F]; e^h_uv = LeakyReLU(<a_src^h, z^h_u> + <a_dst^h, z^h_v>);
 *                    alpha = softmax over u in N(v); h'_v = act(concat_h sum_u alpha^h_uv z^h_u + b)
 *   - Algorithm 2 (Section 2), with one destination node per batch: for l = 1..L, for every v,
 *     compute H^l[v] from H^{l-1}; release H^{l-1} after the layer.
 *
 * Readings where the paper is silent: a sum or mean over an empty N(v) is the zero vector; degrees in
 * the GCN normaliser are counted on the stored CSR (duplicates with multiplicity) and clamped to >= 1;
 * the summation runs in stored CSR order; weights are row-major [in x out] so that h W is a row vector
 * times a matrix.
 *
 * Storage precision: every matrix is passed as float.  With storage == 1 (bf16) the caller passes values
 * already representable in bfloat16 and each stored layer output is rounded to bfloat16
 * (round-to-nearest-even from the double result); with storage == 0 outputs are rounded to float.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC -o libdgi_oracle.so dgi_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { AGG_SUM = 0, AGG_MEAN = 1, AGG_GCN = 2, AGG_GAT = 3 };
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_ELU = 2, ACT_LEAKY = 3 };

typedef struct {
    int agg, act;
    double act_slope;
    int in_dim, out_dim, heads;
    const float* W_self;   /* [in_dim x out_dim] or NULL */
    const float* W_neigh;  /* [in_dim x out_dim] */
    const float* bias;     /* [out_dim] or NULL */
    const float* attn_src; /* [heads x F] (GAT) */
    const float* attn_dst;
    double attn_slope;
    int out_storage;       /* 0 = float, 1 = bfloat16 values held in float */
} oracle_layer_t;

static double activate(double x, int act, double slope) {
    switch (act) {
        case ACT_RELU: return x > 0.0 ? x : 0.0;
        case ACT_ELU: return x > 0.0 ? x : slope * expm1(x);
        case ACT_LEAKY: return x > 0.0 ? x : slope * x;
        default: return x;
    }
}

/* nearest bfloat16 (8 significant bits), ties to even, of a finite double */
static double round_bf16(double x) {
    if (x == 0.0 || !isfinite(x)) return x;
    int e;
    double m = frexp(x, &e);        /* x = m 2^e, 0.5 <= |m| < 1 */
    double q = rint(m * 256.0);     /* default rounding mode: ties to even */
    return ldexp(q / 256.0, e);
}

static float store(double x, int storage) { return (float)(storage == 1 ? round_bf16(x) : x); }

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
void oracle_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* d_out[u] = number of stored edges whose source is u */
void oracle_out_degree(int64_t N, int64_t E, const int32_t* indices, int64_t* d_out) {
    for (int64_t u = 0; u < N; ++u) d_out[u] = 0;
    for (int64_t e = 0; e < E; ++e) d_out[indices[e]] += 1;
}

/* Z[u,:] = H[u,:] W for all u (GAT's per-node projection), kept in double */
static void project_all(int64_t N, int in_dim, int out_dim, const float* H, const float* W, double* Z) {
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < N; ++u) {
        for (int j = 0; j < out_dim; ++j) {
            double s = 0.0;
            for (int k = 0; k < in_dim; ++k) s += (double)H[u * in_dim + k] * (double)W[(int64_t)k * out_dim + j];
            Z[u * out_dim + j] = s;
        }
    }
}

/* One SUM / MEAN / GCN destination row: aggregate in double, then the dense transform. */
static void dense_row(const oracle_layer_t* L, const int64_t* indptr, const int32_t* indices,
                      const int64_t* d_out, const float* H, int64_t v, double* m, float* out_row) {
    const int K = L->in_dim, D = L->out_dim;
    const int64_t a = indptr[v], b = indptr[v + 1];
    for (int k = 0; k < K; ++k) m[k] = 0.0;
    for (int64_t e = a; e < b; ++e) {
        const int64_t u = indices[e];
        double c = 1.0;
        if (L->agg == AGG_GCN) {
            double du = (double)(d_out[u] < 1 ? 1 : d_out[u]);
            double dv = (double)((b - a) < 1 ? 1 : (b - a));
            c = 1.0 / sqrt(du * dv);
        }
        for (int k = 0; k < K; ++k) m[k] += c * (double)H[u * K + k];
    }
    if (L->agg == AGG_MEAN && b > a) {
        for (int k = 0; k < K; ++k) m[k] /= (double)(b - a);
    }
    for (int j = 0; j < D; ++j) {
        double s = L->bias ? (double)L->bias[j] : 0.0;
        for (int k = 0; k < K; ++k) s += m[k] * (double)L->W_neigh[(int64_t)k * D + j];
        if (L->W_self && L->agg != AGG_GCN) {
            for (int k = 0; k < K; ++k) s += (double)H[v * K + k] * (double)L->W_self[(int64_t)k * D + j];
        }
        out_row[j] = store(activate(s, L->act, L->act_slope), L->out_storage);
    }
}

/* One GAT destination row from the projected matrix Z. */
static void gat_row(const oracle_layer_t* L, const int64_t* indptr, const int32_t* indices, const double* Z,
                    int64_t v, double* score, float* out_row) {
    const int D = L->out_dim, Hn = L->heads, F = D / Hn;
    const int64_t a = indptr[v], b = indptr[v + 1];
    for (int h = 0; h < Hn; ++h) {
        double er = 0.0;
        for (int f = 0; f < F; ++f) er += (double)L->attn_dst[h * F + f] * Z[v * D + h * F + f];
        double mx = -INFINITY;
        for (int64_t e = a; e < b; ++e) {
            const int64_t u = indices[e];
            double el = 0.0;
            for (int f = 0; f < F; ++f) el += (double)L->attn_src[h * F + f] * Z[u * D + h * F + f];
            double s = el + er;
            s = s > 0.0 ? s : L->attn_slope * s;
            score[e - a] = s;
            if (s > mx) mx = s;
        }
        double denom = 0.0;
        for (int64_t e = a; e < b; ++e) {
            score[e - a] = exp(score[e - a] - mx);
            denom += score[e - a];
        }
        for (int f = 0; f < F; ++f) {
            double s = 0.0;
            for (int64_t e = a; e < b; ++e) s += (score[e - a] / denom) * Z[(int64_t)indices[e] * D + h * F + f];
            s += L->bias ? (double)L->bias[h * F + f] : 0.0;
            out_row[h * F + f] = store(activate(s, L->act, L->act_slope), L->out_storage);
        }
    }
}

/*
 * One layer of Eq. 1 for the destination rows rows[0..n_rows) (rows == NULL: rows 0..n_rows-1, and then
 * n_rows is normally N).  H_in is the full [N x in_dim] matrix, dense.  Row i of the result is written
 * to H_out[i * out_dim ...] (so with rows == NULL and n_rows == N, H_out is the full next layer).
 * Returns 0, or -1 on a bad argument / allocation failure.
 */
int oracle_layer_forward(int64_t N, const int64_t* indptr, const int32_t* indices, const oracle_layer_t* L,
                         const float* H_in, const int64_t* rows, int64_t n_rows, float* H_out) {
    if (!indptr || !L || !H_out || N < 0 || n_rows < 0) return -1;
    if (N == 0 || n_rows == 0) return 0;
    const int64_t E = indptr[N];
    int64_t max_deg = 0;
    for (int64_t v = 0; v < N; ++v)
        if (indptr[v + 1] - indptr[v] > max_deg) max_deg = indptr[v + 1] - indptr[v];
    int fail = 0;

    if (L->agg == AGG_GAT) {
        if (L->heads < 1 || L->out_dim % L->heads) return -1;
        double* Z = (double*)malloc(sizeof(double) * (size_t)N * L->out_dim);
        if (!Z) return -1;
        project_all(N, L->in_dim, L->out_dim, H_in, L->W_neigh, Z);
#pragma omp parallel
        {
            double* score = (double*)malloc(sizeof(double) * (size_t)(max_deg + 1));
            if (!score) {
#pragma omp atomic write
                fail = 1;
            }
#pragma omp for schedule(dynamic, 64)
            for (int64_t i = 0; i < n_rows; ++i) {
                if (!score) continue;
                const int64_t v = rows ? rows[i] : i;
                gat_row(L, indptr, indices, Z, v, score, H_out + i * L->out_dim);
            }
            free(score);
        }
        free(Z);
        return fail ? -1 : 0;
    }

    int64_t* d_out = NULL;
    if (L->agg == AGG_GCN) {
        d_out = (int64_t*)malloc(sizeof(int64_t) * (size_t)N);
        if (!d_out) return -1;
        oracle_out_degree(N, E, indices, d_out);
    }
#pragma omp parallel
    {
        double* m = (double*)malloc(sizeof(double) * (size_t)(L->in_dim + 1));
        if (!m) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 64)
        for (int64_t i = 0; i < n_rows; ++i) {
            if (!m) continue;
            const int64_t v = rows ? rows[i] : i;
            dense_row(L, indptr, indices, d_out, H_in, v, m, H_out + i * L->out_dim);
        }
        free(m);
    }
    free(d_out);
    return fail ? -1 : 0;
}

/*
 * Algorithm 2 with one destination node per batch: H^0 = X; for l = 1..L: allocate H^l, compute every
 * row from H^{l-1}, release H^{l-1}.  `out` receives H^L ([N x layers[L-1].out_dim]).
 */
int oracle_infer(int64_t N, const int64_t* indptr, const int32_t* indices, const oracle_layer_t* layers,
                 int num_layers, const float* X, float* out) {
    if (num_layers < 1 || !layers || !out) return -1;
    const float* prev = X;
    float* owned_prev = NULL;
    for (int l = 0; l < num_layers; ++l) {
        const oracle_layer_t* L = &layers[l];
        if (l > 0 && L->in_dim != layers[l - 1].out_dim) { free(owned_prev); return -1; }
        float* cur = (l == num_layers - 1) ? out : (float*)malloc(sizeof(float) * (size_t)(N > 0 ? N : 1) * L->out_dim);
        if (!cur) { free(owned_prev); return -1; }
        int rc = oracle_layer_forward(N, indptr, indices, L, prev, NULL, N, cur);
        free(owned_prev); /* H^{l-1} is no longer needed */
        owned_prev = (l == num_layers - 1) ? NULL : cur;
        prev = cur;
        if (rc) { free(owned_prev); return rc; }
    }
    return 0;
}
