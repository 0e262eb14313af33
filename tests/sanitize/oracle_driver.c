/* Runs cases through the CPU oracle (oracle/confu_oracle.c) from a text stream, for a build with AddressSanitizer and
 * UndefinedBehaviorSanitizer.  Input, whitespace separated, one case after the other until end of file:
 *   A M Hq Hkv D P s scale  parent[M] kind[M]  q[M*Hq*D] k[(P+M)*Hkv*D] v[(P+M)*Hkv*D]      tree attention
 *   C T V C temp rule has_draft  target[T*V] (draft[T*V])  token[T] parent[T] uniforms[2T] con_anchor[C]   tree_accept
 * Output: one line per case - "A rc" followed by out[M*Hq*D] and lse[Hq*M] (%.17g), or "C rc" followed by
 * n_accepted final_token final_kind last_node selected_con path[T]. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_tree_attention(int M, int Hq, int Hkv, int D, int P, int s, double scale, const double* q, const double* k,
                          const double* v, const int32_t* parent, const uint8_t* kind, double* out, double* lse);
int oracle_tree_accept(int T, int V, int C, double temp, int rule, const float* target_logits,
                       const float* draft_logits, const int32_t* token, const int32_t* parent, const float* uniforms,
                       const int32_t* con_anchor, int32_t* path, int32_t* n_accepted, int32_t* final_token,
                       int32_t* final_kind, int32_t* last_node, int32_t* selected_con);

static int read_d(double* x, size_t n) { for (size_t i = 0; i < n; ++i) if (scanf("%lf", &x[i]) != 1) return 0; return 1; }
static int read_f(float* x, size_t n) { for (size_t i = 0; i < n; ++i) if (scanf("%f", &x[i]) != 1) return 0; return 1; }
static int read_i(int32_t* x, size_t n) { for (size_t i = 0; i < n; ++i) if (scanf("%d", &x[i]) != 1) return 0; return 1; }

int main(void) {
    char tag[4];
    while (scanf("%3s", tag) == 1) {
        if (tag[0] == 'A') {
            int M, Hq, Hkv, D, P, s;
            double scale;
            if (scanf("%d %d %d %d %d %d %lf", &M, &Hq, &Hkv, &D, &P, &s, &scale) != 7) return 2;
            if (M < 1 || M > 4096 || Hq < 1 || Hkv < 1 || D < 1 || P < 0) return 2;
            const size_t nq = (size_t)M * Hq * D, nk = (size_t)(P + M) * Hkv * D;
            int32_t* parent = malloc(sizeof(int32_t) * M);
            int32_t* kind32 = malloc(sizeof(int32_t) * M);
            uint8_t* kind = malloc(M);
            double *q = malloc(sizeof(double) * nq), *k = malloc(sizeof(double) * nk), *v = malloc(sizeof(double) * nk);
            double *out = malloc(sizeof(double) * nq), *lse = malloc(sizeof(double) * (size_t)Hq * M);
            if (!read_i(parent, M) || !read_i(kind32, M) || !read_d(q, nq) || !read_d(k, nk) || !read_d(v, nk)) return 2;
            for (int i = 0; i < M; ++i) kind[i] = (uint8_t)kind32[i];
            const int rc = oracle_tree_attention(M, Hq, Hkv, D, P, s, scale, q, k, v, parent, kind, out, lse);
            printf("A %d", rc);
            if (rc == 0) {
                for (size_t i = 0; i < nq; ++i) printf(" %.17g", out[i]);
                for (size_t i = 0; i < (size_t)Hq * M; ++i) printf(" %.17g", lse[i]);
            }
            printf("\n");
            free(parent); free(kind32); free(kind); free(q); free(k); free(v); free(out); free(lse);
        } else if (tag[0] == 'C') {
            int T, V, C, rule, has_draft;
            double temp;
            if (scanf("%d %d %d %lf %d %d", &T, &V, &C, &temp, &rule, &has_draft) != 6) return 2;
            if (T < 1 || T > 4096 || V < 1 || C < 0) return 2;
            float *tl = malloc(sizeof(float) * (size_t)T * V), *dl = has_draft ? malloc(sizeof(float) * (size_t)T * V) : NULL;
            int32_t *token = malloc(sizeof(int32_t) * T), *parent = malloc(sizeof(int32_t) * T);
            int32_t *anchor = malloc(sizeof(int32_t) * (C ? C : 1)), *path = malloc(sizeof(int32_t) * T);
            float* un = malloc(sizeof(float) * 2 * T);
            if (!read_f(tl, (size_t)T * V) || (has_draft && !read_f(dl, (size_t)T * V)) || !read_i(token, T) ||
                !read_i(parent, T) || !read_f(un, 2 * (size_t)T) || !read_i(anchor, C)) return 2;
            int32_t n = 0, tok = 0, kind = 0, last = 0, sel = 0;
            const int rc = oracle_tree_accept(T, V, C, temp, rule, tl, dl, token, parent, un, C ? anchor : NULL, path, &n, &tok,
                                              &kind, &last, &sel);
            printf("C %d", rc);
            if (rc == 0) {
                printf(" %d %d %d %d %d", n, tok, kind, last, sel);
                for (int i = 0; i < T; ++i) printf(" %d", path[i]);
            }
            printf("\n");
            free(tl); free(dl); free(token); free(parent); free(anchor); free(path); free(un);
        } else {
            return 2;
        }
    }
    return 0;
}
