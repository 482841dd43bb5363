/* A plain C client of libw2v_shard.so: no Python, no torch -- only the declarations of
 * include/w2v_shard.h and the HIP runtime's C API for device memory.  It runs one dotprod /
 * coeffs / adjust sequence and one fused training step on a small shard and writes every result
 * to a binary file, which the GPU test compares with what the Python binding returns for the same
 * inputs.  Usage: abi_client <output file>
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <hip/hip_runtime_api.h>

#include "../../include/w2v_shard.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 3; } } while (0)
#define CHECK_W2V(x) do { int rc_ = (x); if (rc_ != 0) { \
    fprintf(stderr, "%s: %d %s\n", #x, rc_, w2v_last_error()); return 4; } } while (0)

enum { V = 1000, D = 64, N = 3000, K = 5, T = K + 1 };

int main(int argc, char** argv) {
    if (argc < 2) { fprintf(stderr, "usage: %s <output file>\n", argv[0]); return 2; }
    static uint64_t counts[V];
    static uint32_t in_idx[N], out_idx[N], rows[V];
    static float dots[N * T], coeffs[N * T], U[V * D], W[V * D];
    for (uint32_t w = 0; w < V; ++w) { counts[w] = 1000000u / (w + 1) + 1; rows[w] = w; }
    uint32_t x = 12345u;                               /* small linear congruential generator */
    for (uint32_t p = 0; p < N; ++p) {
        x = x * 1664525u + 1013904223u; in_idx[p] = (x >> 8) % V;
        x = x * 1664525u + 1013904223u; out_idx[p] = ((x >> 8) % V) * ((x >> 8) % V) / V;
    }

    w2v_shard* sh = NULL;
    CHECK_W2V(w2v_shard_create_ex(V, D, 0, D, 77, 1, &sh));
    CHECK_W2V(w2v_shard_set_counts(sh, counts, 0.0));

    uint32_t *d_in, *d_out, *d_rows;
    float *d_dots, *d_coeffs, *d_rowbuf;
    double* d_loss;
    CHECK_HIP(hipMalloc((void**)&d_in, sizeof(in_idx)));
    CHECK_HIP(hipMalloc((void**)&d_out, sizeof(out_idx)));
    CHECK_HIP(hipMalloc((void**)&d_rows, sizeof(rows)));
    CHECK_HIP(hipMalloc((void**)&d_dots, sizeof(dots)));
    CHECK_HIP(hipMalloc((void**)&d_coeffs, sizeof(coeffs)));
    CHECK_HIP(hipMalloc((void**)&d_rowbuf, sizeof(U)));
    CHECK_HIP(hipMalloc((void**)&d_loss, 2 * sizeof(double)));
    CHECK_HIP(hipMemcpy(d_in, in_idx, sizeof(in_idx), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_out, out_idx, sizeof(out_idx), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_rows, rows, sizeof(rows), hipMemcpyHostToDevice));

    hipStream_t st;
    CHECK_HIP(hipStreamCreate(&st));
    const uint64_t seed = w2v_minibatch_seed(99, 0);
    const float* parts[1] = { d_dots };
    CHECK_W2V(w2v_dotprod(sh, d_in, d_out, N, K, seed, d_dots, st));
    CHECK_W2V(w2v_coeffs(sh, parts, 1, N, K, d_coeffs, d_loss, st));
    CHECK_W2V(w2v_adjust(sh, d_in, d_out, N, K, seed, d_coeffs, 0.05f, st));
    CHECK_W2V(w2v_train_minibatch(&sh, 1, d_in, d_out, N, K, w2v_minibatch_seed(99, 1), 0.05f,
                                  d_loss + 1, st));
    CHECK_W2V(w2v_shard_status(sh, st));
    double loss[2];
    CHECK_HIP(hipMemcpy(dots, d_dots, sizeof(dots), hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(coeffs, d_coeffs, sizeof(coeffs), hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(loss, d_loss, sizeof(loss), hipMemcpyDeviceToHost));
    CHECK_W2V(w2v_shard_get_rows(sh, 0, d_rows, V, d_rowbuf, st));
    CHECK_HIP(hipStreamSynchronize(st));
    CHECK_HIP(hipMemcpy(U, d_rowbuf, sizeof(U), hipMemcpyDeviceToHost));
    CHECK_W2V(w2v_shard_get_rows(sh, 1, d_rows, V, d_rowbuf, st));
    CHECK_HIP(hipStreamSynchronize(st));
    CHECK_HIP(hipMemcpy(W, d_rowbuf, sizeof(W), hipMemcpyDeviceToHost));

    /* an argument error comes back as a code and a text, not as a crash */
    if (w2v_dotprod(sh, d_in, d_out, N, W2V_K_MAX + 1, seed, d_dots, st) != W2V_ERR_ARG) return 5;
    if (w2v_last_error()[0] == 0) return 5;

    FILE* f = fopen(argv[1], "wb");
    if (!f) return 6;
    fwrite(in_idx, sizeof(in_idx), 1, f);
    fwrite(out_idx, sizeof(out_idx), 1, f);
    fwrite(dots, sizeof(dots), 1, f);
    fwrite(coeffs, sizeof(coeffs), 1, f);
    fwrite(loss, sizeof(loss), 1, f);
    fwrite(U, sizeof(U), 1, f);
    fwrite(W, sizeof(W), 1, f);
    fclose(f);
    CHECK_W2V(w2v_shard_destroy(sh));
    printf("abi_client ok: loss %.6f %.6f\n", loss[0], loss[1]);
    return 0;
}
