/* Runs every oracle routine on heap buffers that end exactly at the last logical element of the last row, so that an
 * access to row padding after the last row, or past the end, is a heap overflow that AddressSanitizer reports.
 * Built and run by tests/test_oracle_sanitizers.py with -fsanitize=address,undefined.  Test infrastructure. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int gemm_f64_ref(int64_t, int64_t, int64_t, const double *, int64_t, const double *, int64_t, double *, int64_t);
int gemm_f64_ref_ijk(int64_t, int64_t, int64_t, const double *, int64_t, const double *, int64_t, double *, int64_t);
int gemm_f64_absref(int64_t, int64_t, int64_t, const double *, int64_t, const double *, int64_t, double *, int64_t);
int gemm_f32_ref(int64_t, int64_t, int64_t, const float *, int64_t, const float *, int64_t, float *, int64_t);
int gemm_f32_ref_ijk(int64_t, int64_t, int64_t, const float *, int64_t, const float *, int64_t, float *, int64_t);
int gemm_f32_absref(int64_t, int64_t, int64_t, const float *, int64_t, const float *, int64_t, double *, int64_t);
int gemm_f64_general_ref(int, int, int64_t, int64_t, int64_t, double, const double *, int64_t, const double *, int64_t,
                         double, double *, int64_t);
int gemm_f32_general_ref(int, int, int64_t, int64_t, int64_t, float, const float *, int64_t, const float *, int64_t,
                         float, float *, int64_t);

static size_t exact(int64_t rows, int64_t cols, int64_t ld) { return rows > 0 && cols > 0 ? (size_t)((rows - 1) * ld + cols) : 0; }

#define ALLOC(T, name, rows, cols, ld, value)                              \
    size_t name##_n = exact(rows, cols, ld);                               \
    T *name = (T *)malloc((name##_n ? name##_n : 1) * sizeof(T));          \
    for (size_t q = 0; q < name##_n; ++q) name[q] = (T)(value);

static int fails = 0;
#define CHECK(cond, ...) do { if (!(cond)) { fprintf(stderr, __VA_ARGS__); fprintf(stderr, "\n"); ++fails; } } while (0)

static void one_shape(int64_t M, int64_t N, int64_t K, int64_t pa, int64_t pb, int64_t pc)
{
    const int64_t lda = (K > 1 ? K : 1) + pa, ldb = (N > 1 ? N : 1) + pb, ldc = (N > 1 ? N : 1) + pc;
    {   /* plain nests, all-ones data: every logical element of C becomes 1 + K (abs: 1 + K as well) */
        ALLOC(double, A, M, K, lda, 1.0) ALLOC(double, B, K, N, ldb, 1.0) ALLOC(double, C, M, N, ldc, 1.0)
        ALLOC(double, C2, M, N, ldc, 1.0) ALLOC(double, S, M, N, ldc, 1.0)
        CHECK(gemm_f64_ref(M, N, K, A, lda, B, ldb, C, ldc) == 0, "gemm_f64_ref rc");
        CHECK(gemm_f64_ref_ijk(M, N, K, A, lda, B, ldb, C2, ldc) == 0, "gemm_f64_ref_ijk rc");
        CHECK(gemm_f64_absref(M, N, K, A, lda, B, ldb, S, ldc) == 0, "gemm_f64_absref rc");
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j)
                CHECK(C[i * ldc + j] == 1.0 + K && C2[i * ldc + j] == 1.0 + K && S[i * ldc + j] == 1.0 + K, "f64 value at %ld,%ld", (long)i, (long)j);
        free(A); free(B); free(C); free(C2); free(S);
    }
    {
        ALLOC(float, A, M, K, lda, 1.0f) ALLOC(float, B, K, N, ldb, 1.0f) ALLOC(float, C, M, N, ldc, 1.0f)
        ALLOC(float, C2, M, N, ldc, 1.0f) ALLOC(double, S, M, N, ldc, 0.0)
        CHECK(gemm_f32_ref(M, N, K, A, lda, B, ldb, C, ldc) == 0, "gemm_f32_ref rc");
        CHECK(gemm_f32_ref_ijk(M, N, K, A, lda, B, ldb, C2, ldc) == 0, "gemm_f32_ref_ijk rc");
        CHECK(gemm_f32_absref(M, N, K, A, lda, B, ldb, S, ldc) == 0, "gemm_f32_absref rc");
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j)
                CHECK(C[i * ldc + j] == 1.0f + K && C2[i * ldc + j] == 1.0f + K && S[i * ldc + j] == (double)K, "f32 value at %ld,%ld", (long)i, (long)j);
        free(A); free(B); free(C); free(C2); free(S);
    }
    for (int ta = 0; ta < 2; ++ta)
        for (int tb = 0; tb < 2; ++tb) {   /* general form: 2 * K - 3 on all-ones data with alpha = 2, beta = -3 */
            const int64_t ar = ta ? K : M, ac = ta ? M : K, br = tb ? N : K, bc = tb ? K : N;
            const int64_t la = (ac > 1 ? ac : 1) + pa, lb = (bc > 1 ? bc : 1) + pb;
            ALLOC(double, A, ar, ac, la, 1.0) ALLOC(double, B, br, bc, lb, 1.0) ALLOC(double, C, M, N, ldc, 1.0)
            CHECK(gemm_f64_general_ref(ta, tb, M, N, K, 2.0, A, la, B, lb, -3.0, C, ldc) == 0, "general f64 rc");
            ALLOC(float, Af, ar, ac, la, 1.0f) ALLOC(float, Bf, br, bc, lb, 1.0f) ALLOC(float, Cf, M, N, ldc, 1.0f)
            CHECK(gemm_f32_general_ref(ta, tb, M, N, K, 2.0f, Af, la, Bf, lb, -3.0f, Cf, ldc) == 0, "general f32 rc");
            for (int64_t i = 0; i < M; ++i)
                for (int64_t j = 0; j < N; ++j)
                    CHECK(C[i * ldc + j] == 2.0 * K - 3.0 && Cf[i * ldc + j] == 2.0f * K - 3.0f, "general value at %ld,%ld trans %d%d", (long)i, (long)j, ta, tb);
            /* folded forms must not touch A and B at all: pass pointers that may not be dereferenced */
            CHECK(gemm_f64_general_ref(ta, tb, M, N, K, 0.0, NULL, la, NULL, lb, 0.5, C, ldc) == 0, "alpha = 0 rc");
            free(A); free(B); free(C); free(Af); free(Bf); free(Cf);
        }
}

int main(void)
{
    const int64_t shapes[][3] = {{0, 0, 0}, {1, 1, 1}, {0, 5, 3}, {4, 0, 3}, {4, 5, 0}, {3, 5, 7}, {17, 9, 33}, {64, 31, 5}, {2, 70, 19}};
    for (size_t s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s) {
        one_shape(shapes[s][0], shapes[s][1], shapes[s][2], 0, 0, 0);
        one_shape(shapes[s][0], shapes[s][1], shapes[s][2], 3, 1, 2);
    }
    if (fails) { fprintf(stderr, "%d checks failed\n", fails); return 1; }
    puts("oracle sanitizer run ok");
    return 0;
}
