"""The oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only):
a small C driver runs ragged, padded and strided cases through every entry point
(forward, both gradients, their point-wise forms, the plain matrix product) with
exactly-sized heap buffers, so that an index that strays is a hard error."""
import os
import subprocess
import textwrap

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = textwrap.dedent(r"""
    #include <stdint.h>
    #include <stdio.h>
    #include <stdlib.h>
    int mdnn_oracle_out_dims(int, int, int, int, int, int*, int*);
    int mdnn_oracle_conv_fprop(const float*, const float*, float*, double*, int, int, int, int, int,
                               int, int, int, float, int);
    int mdnn_oracle_conv_fprop_points(const float*, const float*, const int32_t*, int64_t, float*, double*,
                                      int, int, int, int, int, int, int, int, float);
    int mdnn_oracle_conv_bprop_data(const float*, const float*, float*, double*, int, int, int, int, int,
                                    int, int, int, float, int);
    int mdnn_oracle_conv_bprop_filter(const float*, const float*, float*, double*, int, int, int, int, int,
                                      int, int, int, float, int);
    int mdnn_oracle_conv_bprop_data_points(const float*, const float*, const int*, long long, float*, double*,
                                           int, int, int, int, int, int, int, int, float);
    int mdnn_oracle_conv_bprop_filter_points(const float*, const float*, const int*, long long, float*, double*,
                                             int, int, int, int, int, int, int, int, float);
    int mdnn_oracle_sgemm_tn(const float*, const float*, float*, double*, int, int, int, float, int);
    /* both gradients and their point-wise entries, exactly-sized heap buffers */
    static int run_gradients(int Nb, int Wi, int Hi, int Nc, int No, int Sk, int s, int p) {
        int Wo, Ho;
        if (mdnn_oracle_out_dims(Wi, Hi, Sk, s, p, &Wo, &Ho)) return 1;
        size_t ni = (size_t)Nc * Hi * Wi * Nb, nf = (size_t)Nc * Sk * Sk * No, no = (size_t)No * Ho * Wo * Nb;
        float* in = malloc(ni * 4); float* f = malloc(nf * 4); float* g = malloc(no * 4);
        float* din = malloc(ni * 4); float* df = malloc(nf * 4);
        double* abi = malloc(ni * 8); double* abf = malloc(nf * 8);
        for (size_t i = 0; i < ni; ++i) in[i] = (float)((i * 7) % 11) - 5.0f;
        for (size_t i = 0; i < nf; ++i) f[i] = (float)((i * 5) % 7) - 3.0f;
        for (size_t i = 0; i < no; ++i) g[i] = (float)((i * 3) % 5) - 2.0f;
        int rc = mdnn_oracle_conv_bprop_data(g, f, din, abi, Nb, Wi, Hi, Nc, No, Sk, s, p, 0.5f, 2);
        rc |= mdnn_oracle_conv_bprop_data(g, f, din, NULL, Nb, Wi, Hi, Nc, No, Sk, s, p, 0.5f, 1);
        rc |= mdnn_oracle_conv_bprop_filter(in, g, df, abf, Nb, Wi, Hi, Nc, No, Sk, s, p, 0.5f, 2);
        rc |= mdnn_oracle_conv_bprop_filter(in, g, df, NULL, Nb, Wi, Hi, Nc, No, Sk, s, p, 0.5f, 1);
        int idx[8] = {0, 0, 0, 0, Nc - 1, Hi - 1, Wi - 1, Nb - 1};
        float v[2]; double a[2];
        rc |= mdnn_oracle_conv_bprop_data_points(g, f, idx, 2, v, a, Nb, Wi, Hi, Nc, No, Sk, s, p, 0.5f);
        rc |= (v[0] != din[0]) || (v[1] != din[ni - 1]);
        int fidx[8] = {0, 0, 0, 0, Nc - 1, Sk - 1, Sk - 1, No - 1};
        rc |= mdnn_oracle_conv_bprop_filter_points(in, g, fidx, 2, v, a, Nb, Wi, Hi, Nc, No, Sk, s, p, 0.5f);
        rc |= (v[0] != df[0]) || (v[1] != df[nf - 1]);
        free(in); free(f); free(g); free(din); free(df); free(abi); free(abf);
        return rc;
    }
    static int run_sgemm(int N, int M, int K) {
        float* a = malloc((size_t)K * N * 4); float* b = malloc((size_t)K * M * 4); float* c = malloc((size_t)N * M * 4);
        double* ab = malloc((size_t)N * M * 8);
        for (int i = 0; i < K * N; ++i) a[i] = (float)((i * 7) % 11) - 5.0f;
        for (int i = 0; i < K * M; ++i) b[i] = (float)((i * 5) % 7) - 3.0f;
        int rc = mdnn_oracle_sgemm_tn(a, b, c, ab, N, M, K, 0.5f, 2);
        rc |= mdnn_oracle_sgemm_tn(a, b, c, NULL, N, M, K, 0.5f, 1);
        free(a); free(b); free(c); free(ab);
        return rc;
    }
    static int run(int Nb, int Wi, int Hi, int Nc, int No, int Sk, int s, int p) {
        int Wo, Ho;
        if (mdnn_oracle_out_dims(Wi, Hi, Sk, s, p, &Wo, &Ho)) return 1;
        size_t ni = (size_t)Nc * Hi * Wi * Nb, nf = (size_t)Nc * Sk * Sk * No, no = (size_t)No * Ho * Wo * Nb;
        float* in = malloc(ni * 4); float* f = malloc(nf * 4); float* out = malloc(no * 4);
        double* ab = malloc(no * 8);
        for (size_t i = 0; i < ni; ++i) in[i] = (float)((i * 7) % 11) - 5.0f;
        for (size_t i = 0; i < nf; ++i) f[i] = (float)((i * 5) % 7) - 3.0f;
        int rc = mdnn_oracle_conv_fprop(in, f, out, ab, Nb, Wi, Hi, Nc, No, Sk, s, p, 0.5f, 2);
        rc |= mdnn_oracle_conv_fprop(in, f, out, NULL, Nb, Wi, Hi, Nc, No, Sk, s, p, 0.5f, 1);
        int32_t idx[8] = {0, 0, 0, 0, No - 1, Ho - 1, Wo - 1, Nb - 1};
        float v[2]; double a[2];
        rc |= mdnn_oracle_conv_fprop_points(in, f, idx, 2, v, a, Nb, Wi, Hi, Nc, No, Sk, s, p, 0.5f);
        rc |= (v[0] != out[0]) || (v[1] != out[no - 1]);
        free(in); free(f); free(out); free(ab);
        return rc;
    }
    int main(void) {
        int rc = 0;
        rc |= run(3, 7, 6, 2, 4, 3, 1, 1);
        rc |= run(5, 9, 4, 3, 2, 5, 2, 2);
        rc |= run(1, 3, 3, 1, 1, 3, 1, 0);
        rc |= run(2, 8, 8, 2, 3, 3, 3, 2);
        rc |= run(4, 11, 5, 1, 5, 1, 1, 0);
        rc |= run_gradients(3, 7, 6, 2, 4, 3, 1, 1);
        rc |= run_gradients(5, 9, 4, 3, 2, 5, 2, 2);
        rc |= run_gradients(1, 3, 3, 1, 1, 3, 1, 0);
        rc |= run_gradients(2, 8, 8, 2, 3, 3, 3, 2);      /* last rows and columns never read */
        rc |= run_gradients(2, 5, 6, 2, 3, 3, 1, 3);      /* pad = Sk */
        rc |= run_gradients(4, 11, 5, 1, 5, 1, 1, 0);
        rc |= run_sgemm(3, 5, 7);
        rc |= run_sgemm(1, 1, 1);
        rc |= run_sgemm(8, 2, 13);
        printf("sanitized oracle rc=%d\n", rc);
        return rc;
    }
""")


def test_oracle_clean_under_asan_ubsan(tmp_path):
    drv = tmp_path / "driver.c"
    exe = tmp_path / "driver"
    drv.write_text(DRIVER)
    subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-o", str(exe), str(drv), os.path.join(ROOT, "oracle", "mdnn_oracle.c"), "-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", OMP_NUM_THREADS="2")
    env.pop("LD_PRELOAD", None)
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env)
    assert res.returncode == 0, res.stdout[-3000:]
    assert "sanitized oracle rc=0" in res.stdout
