/* The hot path from plain C, with no Python or PyTorch in the process: the library creates its own streams and
 * arenas, the program brings page-locked host memory from the HIP runtime's C API, streams every layer in, runs a
 * prefill batch behind the frontier, then one decode step, and writes both outputs to a file.  The GPU test that
 * builds and runs it (tests/test_gpu_boundary.py) prepares the input file from the seeded generators and compares
 * the output file with the oracle.
 *
 * usage: gpu_run <in> <out>
 * <in>:  int32 L, H, Hq, Hkv, d, F, T (prompt tokens of the one sequence); float eps, rope_base;
 *        L layer blobs of bz_sizes.layer_bytes bytes; T*H bf16 hidden states (prefill); H bf16 hidden states (decode)
 * <out>: T*H bf16 (prefill output), H bf16 (decode output)
 * Every layer is also read back and compared with what was sent.  Exit status 0 = everything succeeded. */
#define _POSIX_C_SOURCE 199309L
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include <hip/hip_runtime_api.h>

#include "blitz_layer.h"

#define BZ(call)                                                                                      \
    do {                                                                                              \
        int rc__ = (call);                                                                            \
        if (rc__ != BZ_OK) {                                                                          \
            fprintf(stderr, "line %d: %s -> %s %s\n", __LINE__, #call, bz_strerror(rc__),             \
                    rc__ == BZ_EHIP ? bz_last_hip_error() : "");                                      \
            return 1;                                                                                 \
        }                                                                                             \
    } while (0)
#define HIP(call)                                                                                     \
    do {                                                                                              \
        hipError_t e__ = (call);                                                                      \
        if (e__ != hipSuccess) {                                                                      \
            fprintf(stderr, "line %d: %s -> %s\n", __LINE__, #call, hipGetErrorString(e__));          \
            return 1;                                                                                 \
        }                                                                                             \
    } while (0)

static int read_all(FILE* f, void* dst, size_t n) { return fread(dst, 1, n, f) == n ? 0 : 1; }

static double now_ms(void) {
    struct timespec t;
    clock_gettime(CLOCK_MONOTONIC, &t);
    return (double)t.tv_sec * 1e3 + (double)t.tv_nsec * 1e-6;
}

int main(int argc, char** argv) {
    int32_t hdr[7];
    float fl[2];
    bz_config cfg;
    bz_sizes sz;
    bz_instance* inst = NULL;
    bz_batch *prefill = NULL, *decode = NULL;
    unsigned char *blobs = NULL, *back = NULL;
    void *x_host = NULL, *x_dev = NULL;
    FILE *in, *out;
    int l, T;
    size_t row_bytes;
    const double t_start = now_ms();
    double t_runtime, t_create0, t_created, t_load0, t_done;

    if (argc != 3) { fprintf(stderr, "usage: %s <in> <out>\n", argv[0]); return 2; }
    in = fopen(argv[1], "rb");
    if (!in || read_all(in, hdr, sizeof hdr) || read_all(in, fl, sizeof fl)) { fprintf(stderr, "bad input file\n"); return 2; }

    memset(&cfg, 0, sizeof cfg);                      /* streams and arenas NULL: the library makes its own */
    cfg.n_layers = hdr[0]; cfg.hidden = hdr[1]; cfg.n_q_heads = hdr[2]; cfg.n_kv_heads = hdr[3];
    cfg.head_dim = hdr[4]; cfg.ffn = hdr[5];
    T = hdr[6];
    cfg.rms_eps = fl[0]; cfg.rope_base = fl[1];
    cfg.max_seqs = 1; cfg.max_seq_len = T + 8; cfg.max_tokens = T; cfg.kv_tokens = T + 40;
    BZ(bz_query_sizes(&cfg, &sz));
    if (sz.act_elem_bytes != 2) { fprintf(stderr, "this program feeds bf16 activations\n"); return 2; }
    row_bytes = (size_t)cfg.hidden * 2;

    HIP(hipFree(NULL));                               /* brings the runtime up */
    t_runtime = now_ms();
    HIP(hipHostMalloc((void**)&blobs, sz.layer_bytes * (size_t)cfg.n_layers, hipHostMallocDefault));
    HIP(hipHostMalloc((void**)&back, sz.layer_bytes, hipHostMallocDefault));
    HIP(hipHostMalloc(&x_host, row_bytes * (size_t)(T + 1), hipHostMallocDefault));
    if (read_all(in, blobs, sz.layer_bytes * (size_t)cfg.n_layers) || read_all(in, x_host, row_bytes * (size_t)(T + 1))) {
        fprintf(stderr, "input file too short\n");
        return 2;
    }
    fclose(in);
    HIP(hipMalloc(&x_dev, row_bytes * (size_t)(T + 1)));
    HIP(hipMemcpy(x_dev, x_host, row_bytes * (size_t)(T + 1), hipMemcpyHostToDevice));

    t_create0 = now_ms();
    BZ(bz_create(&cfg, &inst));
    t_created = now_ms();
    BZ(bz_kv_reserve(inst, 0, T + 1));
    {
        int32_t q_start[2], slot[1] = {0}, before[1] = {0};
        bz_batch_desc d;
        q_start[0] = 0; q_start[1] = T;
        d.n_seqs = 1; d.q_start = q_start; d.seq_slot = slot; d.kv_len_before = before;
        BZ(bz_batch_create(&d, &prefill));
        q_start[1] = 1; before[0] = T;
        BZ(bz_batch_create(&d, &decode));
    }
    /* the run is enqueued first and every layer requested afterwards: execution follows the frontier */
    if (bz_run_layers(inst, 0, cfg.n_layers, prefill, x_dev, 0) != BZ_ENOTLOADED) {
        fprintf(stderr, "a run over layers that were never requested must be refused\n");
        return 1;
    }
    t_load0 = now_ms();
    for (l = 0; l < cfg.n_layers; ++l) BZ(bz_load_layer(inst, l, blobs + sz.layer_bytes * (size_t)l, sz.layer_bytes));
    BZ(bz_run_layers(inst, 0, cfg.n_layers, prefill, x_dev, 0));
    BZ(bz_run_layers(inst, 0, cfg.n_layers, decode, (unsigned char*)x_dev + row_bytes * (size_t)T, 0));
    BZ(bz_sync(inst));
    t_done = now_ms();
    if (bz_frontier(inst) != cfg.n_layers) { fprintf(stderr, "frontier %d\n", bz_frontier(inst)); return 1; }
    for (l = 0; l < cfg.n_layers; ++l) {
        BZ(bz_readback_layer(inst, l, back));
        if (memcmp(back, blobs + sz.layer_bytes * (size_t)l, sz.layer_bytes) != 0) {
            fprintf(stderr, "layer %d differs from the host copy\n", l);
            return 1;
        }
    }
    HIP(hipMemcpy(x_host, x_dev, row_bytes * (size_t)(T + 1), hipMemcpyDeviceToHost));
    out = fopen(argv[2], "wb");
    if (!out || fwrite(x_host, 1, row_bytes * (size_t)(T + 1), out) != row_bytes * (size_t)(T + 1) || fclose(out)) {
        fprintf(stderr, "cannot write %s\n", argv[2]);
        return 2;
    }
    BZ(bz_batch_destroy(prefill));
    BZ(bz_batch_destroy(decode));
    BZ(bz_destroy(inst));
    HIP(hipFree(x_dev));
    HIP(hipHostFree(x_host));
    HIP(hipHostFree(back));
    HIP(hipHostFree(blobs));
    printf("ran %d layers over %d prompt tokens and one decode step\n", (int)cfg.n_layers, T);
    printf("runtime up after %.0f ms; bz_create %.1f ms; first load request to both outputs %.1f ms (first use of the "
           "kernels included)\n", t_runtime - t_start, t_created - t_create0, t_done - t_load0);
    return 0;
}
