/*
 * Brute-force C twin of the float64 oracle: routed causal grouped-query attention by plain loops.
 *
 * TEST INFRASTRUCTURE ONLY.  It exists so that the numpy oracle can be cross-checked against an
 * independent implementation in another language (scalar loops instead of matrix products), and
 * it shares no code with the HIP library.
 *
 * Follows the paper's Eq. (3.1) (layer l attends to K, V of a source layer l' <= l), Eq. (3.2)
 * (source = nearest preceding cached layer; here the route is given and only validated) and
 * Sec. 3.1.1 (pre-fill of several rows, sampling of one row).  Attn is softmax(scale q K^T) V,
 * query at absolute position p sees keys 0..p, query head h reads kv head h / G.
 *
 * Build: gcc -O2 -fPIC -shared -o libskv_oracle_brute.so skv_oracle_brute.c -lm
 */
#include <math.h>
#include <stdlib.h>

/* slot_of_layer[l] = rank of route[l] among the layers with route[l] == l.
 * Returns 0 if the route is valid, 1 otherwise (outputs then undefined). */
int skvo_slot_map(const int *route, int n_layers, int *slot_of_layer, int *n_slots) {
    if (n_layers <= 0) return 1;
    for (int l = 0; l < n_layers; ++l) {
        if (route[l] < 0 || route[l] > l) return 1;
        if (route[route[l]] != route[l]) return 1;
    }
    int count = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (route[l] == l) {
            slot_of_layer[l] = count++;
        } else {
            slot_of_layer[l] = slot_of_layer[route[l]]; /* route[l] < l: already set */
        }
    }
    *n_slots = count;
    return 0;
}

/*
 * kc, vc : [n_slots][batch][ctx][kv_heads][d]   logical cache, float64
 * q, out : [batch][max_q][q_heads][d]
 * Row i < q_lens[b] of sequence b sits at absolute position kv_lens[b] - q_lens[b] + i.
 * Rows i >= q_lens[b] of out are left untouched.  Returns 0 on success.
 */
int skvo_attention(const double *kc, const double *vc, int batch, int ctx, int kv_heads, int d,
                   int slot, const double *q, int max_q, int q_heads, const int *q_lens,
                   const int *kv_lens, double scale, double *out) {
    if (q_heads % kv_heads) return 1;
    const int G = q_heads / kv_heads;
    double *w = (double *)malloc(sizeof(double) * (size_t)(ctx > 0 ? ctx : 1));
    if (!w) return 2;
    for (int b = 0; b < batch; ++b) {
        if (q_lens[b] > kv_lens[b] || kv_lens[b] > ctx || q_lens[b] > max_q) { free(w); return 1; }
        for (int i = 0; i < q_lens[b]; ++i) {
            const int p = kv_lens[b] - q_lens[b] + i;
            for (int h = 0; h < q_heads; ++h) {
                const int kvh = h / G;
                const double *qv = q + (((size_t)b * max_q + i) * q_heads + h) * d;
                double *ov = out + (((size_t)b * max_q + i) * q_heads + h) * d;
                double m = -INFINITY;
                for (int j = 0; j <= p; ++j) {
                    const double *kr =
                        kc + ((((size_t)slot * batch + b) * ctx + j) * kv_heads + kvh) * d;
                    double s = 0.0;
                    for (int e = 0; e < d; ++e) s += qv[e] * kr[e];
                    w[j] = s * scale;
                    if (w[j] > m) m = w[j];
                }
                double z = 0.0;
                for (int j = 0; j <= p; ++j) {
                    w[j] = exp(w[j] - m);
                    z += w[j];
                }
                for (int e = 0; e < d; ++e) ov[e] = 0.0;
                for (int j = 0; j <= p; ++j) {
                    const double *vr =
                        vc + ((((size_t)slot * batch + b) * ctx + j) * kv_heads + kvh) * d;
                    const double pj = w[j] / z;
                    for (int e = 0; e < d; ++e) ov[e] += pj * vr[e];
                }
            }
        }
    }
    free(w);
    return 0;
}
