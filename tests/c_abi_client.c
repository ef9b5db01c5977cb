/* A client of libsamp written in plain C99: shows that the boundary needs nothing but include/samp.h,
 * plain pointers and the HIP runtime's C API for device memory.
 *
 * usage: c_abi_client <in.bin> <out.bin>
 * in.bin (little endian, written by tests/test_c_client.py):
 *   int32 layers, hidden, heads, ffn, B, S, has_mask;  float ln_eps;
 *   uint8 modes[layers];
 *   per layer: w_qkv, w_o, w_ffn1, w_ffn2 (fp16), b_qkv, b_o, b_ffn1, b_ffn2, ln1_g, ln1_b, ln2_g, ln2_b (float);
 *   float scales[layers][10];  fp16 hidden[B*S*hidden];  int32 mask[B*S] if has_mask.
 * out.bin: fp16 out[B*S*hidden] of samp_encoder_forward, called twice (the second call replays the recorded graph)
 * and compared here byte for byte.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "samp.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_SAMP(x) do { int rc_ = (x); if (rc_ != SAMP_OK) { fprintf(stderr, "%s: %d %s\n", #x, rc_, samp_last_error()); return 3; } } while (0)

static void *take(FILE *f, size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) { fprintf(stderr, "short input file\n"); exit(4); }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3) { fprintf(stderr, "usage: %s in.bin out.bin\n", argv[0]); return 1; }
    FILE *f = fopen(argv[1], "rb");
    if (!f) { perror(argv[1]); return 1; }
    int32_t *hd = (int32_t *)take(f, 7 * sizeof(int32_t));
    const int32_t layers = hd[0], H = hd[1], heads = hd[2], F = hd[3], B = hd[4], S = hd[5], has_mask = hd[6];
    float *eps = (float *)take(f, sizeof(float));
    uint8_t *modes = (uint8_t *)take(f, (size_t)layers);
    samp_layer_weights_t *w = (samp_layer_weights_t *)calloc((size_t)layers, sizeof(*w));
    for (int l = 0; l < layers; l++) {
        w[l].w_qkv = (const uint16_t *)take(f, (size_t)3 * H * H * 2);
        w[l].w_o = (const uint16_t *)take(f, (size_t)H * H * 2);
        w[l].w_ffn1 = (const uint16_t *)take(f, (size_t)F * H * 2);
        w[l].w_ffn2 = (const uint16_t *)take(f, (size_t)H * F * 2);
        w[l].b_qkv = (const float *)take(f, (size_t)3 * H * 4);
        w[l].b_o = (const float *)take(f, (size_t)H * 4);
        w[l].b_ffn1 = (const float *)take(f, (size_t)F * 4);
        w[l].b_ffn2 = (const float *)take(f, (size_t)H * 4);
        w[l].ln1_g = (const float *)take(f, (size_t)H * 4);
        w[l].ln1_b = (const float *)take(f, (size_t)H * 4);
        w[l].ln2_g = (const float *)take(f, (size_t)H * 4);
        w[l].ln2_b = (const float *)take(f, (size_t)H * 4);
    }
    samp_layer_scales_t *sc = (samp_layer_scales_t *)take(f, (size_t)layers * sizeof(samp_layer_scales_t));
    const size_t n_act = (size_t)B * S * H;
    uint16_t *hidden = (uint16_t *)take(f, n_act * 2);
    int32_t *mask = has_mask ? (int32_t *)take(f, (size_t)B * S * 4) : NULL;
    fclose(f);

    samp_config_t cfg;
    memset(&cfg, 0, sizeof(cfg));
    cfg.layers = layers; cfg.hidden = H; cfg.heads = heads; cfg.ffn = F; cfg.max_batch = B; cfg.max_seq = S; cfg.ln_eps = *eps;

    const size_t arena_bytes = samp_encoder_arena_bytes(&cfg, modes);
    if (!arena_bytes) { fprintf(stderr, "arena_bytes: %s\n", samp_last_error()); return 3; }
    void *arena = NULL, *ws = NULL, *d_hidden = NULL, *d_out = NULL, *d_mask = NULL;
    CHECK_HIP(hipMalloc(&arena, arena_bytes));
    samp_encoder_t *enc = NULL;
    CHECK_SAMP(samp_encoder_create(&cfg, modes, w, sc, arena, arena_bytes, NULL, &enc));
    const size_t ws_bytes = samp_encoder_workspace_bytes(enc, B, S);
    CHECK_HIP(hipMalloc(&ws, ws_bytes));
    CHECK_HIP(hipMalloc(&d_hidden, n_act * 2));
    CHECK_HIP(hipMalloc(&d_out, n_act * 2));
    CHECK_HIP(hipMemcpy(d_hidden, hidden, n_act * 2, hipMemcpyHostToDevice));
    if (mask) {
        CHECK_HIP(hipMalloc(&d_mask, (size_t)B * S * 4));
        CHECK_HIP(hipMemcpy(d_mask, mask, (size_t)B * S * 4, hipMemcpyHostToDevice));
    }
    uint16_t *out[3];
    for (int call = 0; call < 3; call++) {          /* plain launches, graph capture, graph replay */
        out[call] = (uint16_t *)malloc(n_act * 2);
        CHECK_HIP(hipMemset(d_out, 0x5a, n_act * 2));
        CHECK_SAMP(samp_encoder_forward(enc, d_hidden, (const int32_t *)d_mask, B, S, d_out, ws, ws_bytes, NULL));
        CHECK_HIP(hipDeviceSynchronize());
        CHECK_HIP(hipMemcpy(out[call], d_out, n_act * 2, hipMemcpyDeviceToHost));
        if (call && memcmp(out[0], out[call], n_act * 2) != 0) { fprintf(stderr, "call %d differs from call 0\n", call); return 5; }
    }
    /* an argument error must come back as a code and a message, not as a crash */
    if (samp_encoder_forward(enc, d_hidden, NULL, B + 1, S, d_out, ws, ws_bytes, NULL) != SAMP_ERR_SHAPE || !samp_last_error()[0]) {
        fprintf(stderr, "expected SAMP_ERR_SHAPE for B above max_batch\n");
        return 6;
    }
    CHECK_SAMP(samp_encoder_destroy(enc));
    f = fopen(argv[2], "wb");
    if (!f || fwrite(out[0], 2, n_act, f) != n_act) { perror(argv[2]); return 1; }
    fclose(f);
    CHECK_HIP(hipFree(arena)); CHECK_HIP(hipFree(ws)); CHECK_HIP(hipFree(d_hidden)); CHECK_HIP(hipFree(d_out));
    if (d_mask) CHECK_HIP(hipFree(d_mask));
    printf("ok %zu values\n", n_act);
    return 0;
}
