/* Driver for the sanitizer build of the CPU oracle (tests/test_sanitizers.py): a small residual network with a
   convolution, an average pooling and dense layers, analysed in every mode of the oracle.  Built together with
   oracle/deeppoly_oracle.c under -fsanitize=address,undefined; any finding aborts with a non-zero status. */
#include <stdio.h>
#include <stdlib.h>

typedef struct dp_net dp_net;
dp_net *dp_create(int c, int h, int w);
void dp_destroy(dp_net *N);
int dp_add_dense(dp_net *N, int src, int n_out, const float *W, const float *b);
int dp_add_conv2d(dp_net *N, int src, int c_out, int kh, int kw, int sh, int sw, int ph, int pw, const float *W, const float *b);
int dp_add_avgpool2d(dp_net *N, int src, int kh, int kw, int sh, int sw, int ph, int pw);
int dp_add_relu(dp_net *N, int src);
int dp_add_residual(dp_net *N, int a, int b);
int dp_layer_size(const dp_net *N, int lid);
int dp_num_layers(const dp_net *N);
int dp_set_options(dp_net *N, int lambda_policy, int candidates);
int dp_set_collapse(dp_net *N, int on);
int dp_set_early_termination(dp_net *N, int on);
int dp_set_float_inference(dp_net *N, int on);
int dp_request_bounds(dp_net *N, int lid);
int dp_set_ball(dp_net *N, const float *center, float eps, float clip_lo, float clip_hi);
int dp_analyze(dp_net *N);
int dp_get_bounds(const dp_net *N, int lid, double *lo, double *hi);
int dp_bound_rows(dp_net *N, int lid, const int *rows, int n_rows, double *out_lo, double *out_hi);
int dp_certify(dp_net *N, int label, int *verified, double *margins);
int dp_bound_forms(dp_net *N, int n_forms, const double *coef, const double *offset, double *lower);
int dp_get_term_layer(const dp_net *N, int lid, int *term);

static unsigned long long state = 12345;
static float rnd(void) {           /* small deterministic generator: values in (-0.5, 0.5) */
    state = state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (float)((state >> 33) % 10001) / 10000.0f - 0.5f;
}
static float *weights(int n, float scale) {
    float *w = (float *)malloc(sizeof(float) * n);
    for (int i = 0; i < n; ++i) w[i] = rnd() * scale;
    return w;
}
#define CHECK(x) do { int rc_ = (x); if (rc_ != 0) { fprintf(stderr, "mode %d: %s -> %d\n", mode, #x, rc_); return 1; } } while (0)

int main(void) {
    dp_net *N = dp_create(2, 8, 8);
    float *w1 = weights(4 * 2 * 3 * 3, 0.6f), *b1 = weights(4, 0.2f);
    int c1 = dp_add_conv2d(N, 0, 4, 3, 3, 1, 1, 1, 1, w1, b1);
    int r1 = dp_add_relu(N, c1);
    float *w2 = weights(4 * 4 * 3 * 3, 0.4f), *b2 = weights(4, 0.2f);
    int c2 = dp_add_conv2d(N, r1, 4, 3, 3, 1, 1, 1, 1, w2, b2);
    int r2 = dp_add_relu(N, c2);
    float *w3 = weights(4 * 4 * 3 * 3, 0.1f);
    int c3 = dp_add_conv2d(N, r2, 4, 3, 3, 1, 1, 1, 1, w3, NULL);
    int s1 = dp_add_residual(N, c3, r1);
    int r3 = dp_add_relu(N, s1);
    int p1 = dp_add_avgpool2d(N, r3, 3, 3, 2, 2, 1, 1);
    int np = dp_layer_size(N, p1);
    float *w4 = weights(6 * np, 0.3f), *b4 = weights(6, 0.1f);
    int d1 = dp_add_dense(N, p1, 6, w4, b4);
    int r4 = dp_add_relu(N, d1);
    float *w5 = weights(3 * 6, 0.5f);
    int out = dp_add_dense(N, r4, 3, w5, NULL);
    if (out != dp_num_layers(N) - 1 || out < 0) return 2;
    /* the dense layer reads the pooling layer directly: its intervals are needed for the float32-inference constants */
    if (dp_request_bounds(N, p1) != 0) return 2;
    float center[128];
    for (int i = 0; i < 128; ++i) center[i] = rnd() + 0.5f;
    double lo[256], hi[256], m[2], forms[6] = {1, -1, 0, 0.5, 0.25, -2}, off[2] = {0.1, -0.3}, lb[2];
    int rows[3] = {0, 5, 3}, verified = 0, term[256];
    for (int mode = 0; mode < 6; ++mode) {
        CHECK(dp_set_collapse(N, mode != 1));
        CHECK(dp_set_early_termination(N, mode == 2 || mode == 4));
        CHECK(dp_set_float_inference(N, mode == 3 || mode == 4));
        CHECK(dp_set_options(N, mode == 5 ? 1 : 0, mode == 5 ? 1 : 0));
        CHECK(dp_set_ball(N, center, 0.03f, 0.0f, 1.0f));
        if (mode == 5) CHECK(dp_request_bounds(N, c3));
        CHECK(dp_analyze(N));
        CHECK(dp_get_bounds(N, out, lo, hi));
        for (int i = 0; i < 3; ++i)
            if (!(lo[i] <= hi[i])) { fprintf(stderr, "mode %d: empty interval\n", mode); return 3; }
        CHECK(dp_get_bounds(N, c2, lo, hi));
        if (mode != 2 && mode != 4) CHECK(dp_bound_rows(N, d1, rows, 3, lo, hi));
        if (mode == 2 || mode == 4) CHECK(dp_get_term_layer(N, c2, term));
        CHECK(dp_certify(N, 1, &verified, m));
        CHECK(dp_bound_forms(N, 2, forms, off, lb));
    }
    dp_destroy(N);
    free(w1); free(b1); free(w2); free(b2); free(w3); free(w4); free(b4); free(w5);
    printf("oracle sanitizer driver: ok\n");
    return 0;
}
