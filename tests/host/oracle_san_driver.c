/* Runs single calls of the CPU oracle in a process of its own, so that the
 * oracle's C files can be checked under AddressSanitizer and
 * UndefinedBehaviorSanitizer (tests/test_oracle_sanitized.py builds this file
 * together with oracle/ *.c with -fsanitize=address,undefined).  Every array is
 * read from a raw file into a heap block of exactly its size and every output
 * goes to a heap block of exactly its size, so an access outside any of them
 * ends the run.
 *
 *   driver conv N C H W O K stride pad  x.i8 w.i8 thr.i32  y.i32 bits.i8 packed.u32 unpacked.i8
 *   driver branches N C H W O F P stride pad shared  xb.i8 padv.i8 w.i8 g.f32 h.f32  z64.f64 z32.f32
 *   driver module ROWS O  y.i32 g.f32 b.f32 id.f32 a.f32 c.f32  r64.f64 r32.f32 bits.i8
 *   driver pool N H W C S  a.f32  p64.f64 p32.f32
 *   driver store COUNT  x.f32  f16.u16 f16back.f32 bf16.u16 bf16back.f32 bf16load.f32
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_out_dim(int in, int k, int stride, int pad);
int oracle_conv2d_pm1(const int8_t *x, const int8_t *w, int N, int C, int H, int W, int O, int KH, int KW,
                      int stride, int pad, int32_t *y);
void oracle_threshold_sign(const int32_t *y, const int32_t *thr, int64_t rows, int O, int8_t *s);
void oracle_pack_channels(const int8_t *s, int64_t outer, int64_t C, int64_t inner, uint32_t *dst);
void oracle_unpack_channels(const uint32_t *src, int64_t outer, int64_t C, int64_t inner, int8_t *s);
void oracle_sign_bias_f32(const float *x, const float *bias, int64_t outer, int64_t C, int64_t inner, int8_t *s);
int oracle_branches_pm1(const int8_t *xb, int shared, const int8_t *padv, const int8_t *w, const float *g,
                        const float *h, int N, int C, int H, int W, int O, int F, int P, int stride, int pad,
                        double *z64, float *z32, int32_t *y_taps);
void oracle_module_epilogue(const int32_t *y, const float *gamma, const float *beta, const float *identity,
                            const float *alpha, int64_t rows, int O, double *r64, float *r32);
int oracle_avgpool_nhwc(const float *a, int N, int H, int W, int C, int S, double *p64, float *p32);
void oracle_store_f16(const float *x, int64_t count, uint16_t *code, float *back);
void oracle_store_bf16(const float *x, int64_t count, uint16_t *code, float *back);
void oracle_load_bf16(const uint16_t *code, int64_t count, float *value);

static void *read_exact(const char *path, size_t bytes)
{
    FILE *f = fopen(path, "rb");
    if (!f) { fprintf(stderr, "cannot open %s\n", path); exit(2); }
    void *p = malloc(bytes ? bytes : 1);
    if (fread(p, 1, bytes, f) != bytes || fgetc(f) != EOF) { fprintf(stderr, "%s: size is not %zu\n", path, bytes); exit(2); }
    fclose(f);
    return p;
}

static void write_out(const char *path, const void *p, size_t bytes)
{
    FILE *f = fopen(path, "wb");
    if (!f || fwrite(p, 1, bytes, f) != bytes) { fprintf(stderr, "cannot write %s\n", path); exit(2); }
    fclose(f);
}

int main(int argc, char **argv)
{
    if (argc < 2) return 2;
    char **a = argv + 2;
    if (!strcmp(argv[1], "conv") && argc == 17) {
        const int N = atoi(a[0]), C = atoi(a[1]), H = atoi(a[2]), W = atoi(a[3]), O = atoi(a[4]), K = atoi(a[5]);
        const int stride = atoi(a[6]), pad = atoi(a[7]);
        const int Ho = oracle_out_dim(H, K, stride, pad), Wo = oracle_out_dim(W, K, stride, pad);
        const size_t rows = (size_t)N * Ho * Wo, cw = (size_t)(O + 31) / 32;
        int8_t *x = read_exact(a[8], (size_t)N * C * H * W), *w = read_exact(a[9], (size_t)O * C * K * K);
        int32_t *thr = read_exact(a[10], 4 * (size_t)O);
        int32_t *y = malloc(4 * rows * O);
        int8_t *s = malloc(rows * O), *t = malloc(rows * O), *u = malloc(rows * O);
        uint32_t *packed = malloc(4 * rows * cw);
        if (oracle_conv2d_pm1(x, w, N, C, H, W, O, K, K, stride, pad, y) != 0) return 3;
        oracle_threshold_sign(y, thr, (int64_t)rows, O, s);
        /* [n][pixel][o] -> [n][o][pixel], the packer's [outer][C][inner] */
        for (int n = 0; n < N; ++n)
            for (size_t p = 0; p < (size_t)Ho * Wo; ++p)
                for (int o = 0; o < O; ++o)
                    t[((size_t)n * O + o) * Ho * Wo + p] = s[((size_t)n * Ho * Wo + p) * O + o];
        oracle_pack_channels(t, N, O, (int64_t)Ho * Wo, packed);
        oracle_unpack_channels(packed, N, O, (int64_t)Ho * Wo, u);
        write_out(a[11], y, 4 * rows * O);
        write_out(a[12], s, rows * O);
        write_out(a[13], packed, 4 * rows * cw);
        write_out(a[14], u, rows * O);
        free(x); free(w); free(thr); free(y); free(s); free(t); free(u); free(packed);
        return 0;
    }
    if (!strcmp(argv[1], "branches") && argc == 19) {
        const int N = atoi(a[0]), C = atoi(a[1]), H = atoi(a[2]), W = atoi(a[3]), O = atoi(a[4]), F = atoi(a[5]);
        const int P = atoi(a[6]), stride = atoi(a[7]), pad = atoi(a[8]), shared = atoi(a[9]);
        const int Ho = oracle_out_dim(H, F, stride, pad), Wo = oracle_out_dim(W, F, stride, pad);
        const size_t outs = (size_t)N * Ho * Wo * O;
        int8_t *xb = read_exact(a[10], (size_t)(shared ? 1 : P) * N * C * H * W);
        int8_t *padv = read_exact(a[11], (size_t)P * C), *w = read_exact(a[12], (size_t)O * C * P);
        float *g = read_exact(a[13], 4 * (size_t)P * O), *h = read_exact(a[14], 4 * (size_t)O);
        double *z64 = malloc(8 * outs);
        float *z32 = malloc(4 * outs);
        if (oracle_branches_pm1(xb, shared, padv, w, g, h, N, C, H, W, O, F, P, stride, pad, z64, z32, NULL) != 0) return 3;
        write_out(a[15], z64, 8 * outs);
        write_out(a[16], z32, 4 * outs);
        free(xb); free(padv); free(w); free(g); free(h); free(z64); free(z32);
        return 0;
    }
    if (!strcmp(argv[1], "module") && argc == 13) {
        const size_t rows = (size_t)atoll(a[0]);
        const int O = atoi(a[1]);
        int32_t *y = read_exact(a[2], 4 * rows * O);
        float *g = read_exact(a[3], 4 * (size_t)O), *b = read_exact(a[4], 4 * (size_t)O);
        float *id = read_exact(a[5], 4 * rows * O), *al = read_exact(a[6], 4 * (size_t)O), *c = read_exact(a[7], 4 * (size_t)O);
        double *r64 = malloc(8 * rows * O);
        float *r32 = malloc(4 * rows * O);
        int8_t *bits = malloc(rows * O);
        oracle_module_epilogue(y, g, b, id, al, (int64_t)rows, O, r64, r32);
        oracle_sign_bias_f32(r32, c, (int64_t)rows, O, 1, bits);
        write_out(a[8], r64, 8 * rows * O);
        write_out(a[9], r32, 4 * rows * O);
        write_out(a[10], bits, rows * O);
        free(y); free(g); free(b); free(id); free(al); free(c); free(r64); free(r32); free(bits);
        return 0;
    }
    if (!strcmp(argv[1], "pool") && argc == 10) {
        const int N = atoi(a[0]), H = atoi(a[1]), W = atoi(a[2]), C = atoi(a[3]), S = atoi(a[4]);
        const size_t outs = (size_t)N * (H / S) * (W / S) * C;
        float *src = read_exact(a[5], 4 * (size_t)N * H * W * C);
        double *p64 = malloc(8 * outs);
        float *p32 = malloc(4 * outs);
        if (oracle_avgpool_nhwc(src, N, H, W, C, S, p64, p32) != 0) return 3;
        write_out(a[6], p64, 8 * outs);
        write_out(a[7], p32, 4 * outs);
        free(src); free(p64); free(p32);
        return 0;
    }
    if (!strcmp(argv[1], "store") && argc == 9) {
        const size_t n = (size_t)atoll(a[0]);
        float *x = read_exact(a[1], 4 * n);
        uint16_t *h = malloc(2 * n), *bf = malloc(2 * n);
        float *hb = malloc(4 * n), *bfb = malloc(4 * n), *bfl = malloc(4 * n);
        oracle_store_f16(x, (int64_t)n, h, hb);
        oracle_store_bf16(x, (int64_t)n, bf, bfb);
        oracle_load_bf16(bf, (int64_t)n, bfl);
        write_out(a[2], h, 2 * n);
        write_out(a[3], hb, 4 * n);
        write_out(a[4], bf, 2 * n);
        write_out(a[5], bfb, 4 * n);
        write_out(a[6], bfl, 4 * n);
        free(x); free(h); free(bf); free(hb); free(bfb); free(bfl);
        return 0;
    }
    fprintf(stderr, "bad command line\n");
    return 2;
}
