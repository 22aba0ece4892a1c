/*
 * A caller of the library written in plain C: no Python, no PyTorch.  It reads a
 * layer and a batch from raw files, places them in device memory with the HIP
 * runtime, runs sere_moe_decode and sere_moe_decode_baseline on a stream of its
 * own and writes the results back as raw files.  The tests use it to show that
 * the boundary in include/sere.h is usable as it is declared, from C.
 *
 *   abi_cli DIR
 *
 * DIR/config.txt: "T d_h M K d_m n_sh dtype S rho flags" (one line).
 * Inputs (raw, little endian, element type of dtype unless noted): hidden.bin,
 * router_w.bin, w_gate_up.bin, w_down.bin, shared_gate_up.bin and
 * shared_down.bin (if n_sh > 0), sim.bin (fp32).
 * Outputs: out.bin, out_baseline.bin (dtype); topk_ids.bin, rerouted_ids.bin,
 * count_before.bin, count_after.bin, primary_mask.bin, num_active.bin,
 * sorted_token.bin, sorted_slot.bin, expert_offsets.bin (int32);
 * topk_weights.bin (fp32) -- all from the sere_moe_decode call.
 * Exit status 0 on success; otherwise a message on stderr and status 1.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sere.h"

#define MAX_BUFFERS 32
static void *g_device[MAX_BUFFERS];
static int g_num_device = 0;

static void fail(const char *what, const char *detail)
{
    fprintf(stderr, "abi_cli: %s: %s\n", what, detail);
    exit(1);
}

static void check_hip(hipError_t e, const char *what)
{
    if (e != hipSuccess)
        fail(what, hipGetErrorString(e));
}

static void check_sere(int status, const char *what)
{
    if (status != SERE_OK)
        fail(what, sere_status_string(status));
}

static void *device_alloc(size_t bytes)
{
    void *p = NULL;
    if (g_num_device == MAX_BUFFERS)
        fail("device_alloc", "too many buffers");
    check_hip(hipMalloc(&p, bytes > 0 ? bytes : 1), "hipMalloc");
    g_device[g_num_device++] = p;
    return p;
}

/* file DIR/name of exactly `bytes` bytes -> new device buffer */
static void *upload(const char *dir, const char *name, size_t bytes)
{
    char path[1024];
    snprintf(path, sizeof path, "%s/%s", dir, name);
    FILE *f = fopen(path, "rb");
    if (f == NULL)
        fail("cannot open", path);
    void *host = malloc(bytes > 0 ? bytes : 1);
    if (host == NULL)
        fail("malloc", path);
    if (fread(host, 1, bytes, f) != bytes || fgetc(f) != EOF)
        fail("wrong size", path);
    fclose(f);
    void *dev = device_alloc(bytes);
    check_hip(hipMemcpy(dev, host, bytes, hipMemcpyHostToDevice), "hipMemcpy to device");
    free(host);
    return dev;
}

/* device buffer -> file DIR/name */
static void download(const char *dir, const char *name, const void *dev, size_t bytes)
{
    char path[1024];
    snprintf(path, sizeof path, "%s/%s", dir, name);
    void *host = malloc(bytes > 0 ? bytes : 1);
    if (host == NULL)
        fail("malloc", path);
    check_hip(hipMemcpy(host, dev, bytes, hipMemcpyDeviceToHost), "hipMemcpy to host");
    FILE *f = fopen(path, "wb");
    if (f == NULL)
        fail("cannot create", path);
    if (fwrite(host, 1, bytes, f) != bytes)
        fail("short write", path);
    fclose(f);
    free(host);
}

int main(int argc, char **argv)
{
    if (argc != 2)
        fail("usage", "abi_cli DIR");
    const char *dir = argv[1];
    char path[1024];
    snprintf(path, sizeof path, "%s/config.txt", dir);
    FILE *f = fopen(path, "r");
    if (f == NULL)
        fail("cannot open", path);
    sere_config cfg;
    memset(&cfg, 0, sizeof cfg);
    int fields = fscanf(f, "%d %d %d %d %d %d %d %d %f %d", &cfg.num_tokens, &cfg.hidden,
                        &cfg.num_experts, &cfg.top_k, &cfg.inter, &cfg.num_shared, &cfg.dtype,
                        &cfg.select_top_k, &cfg.threshold, &cfg.flags);
    fclose(f);
    if (fields != 10)
        fail("malformed", path);

    const size_t ws_bytes = sere_workspace_bytes(&cfg);
    if (ws_bytes == 0)
        fail("sere_workspace_bytes", "configuration rejected");
    const size_t eb = cfg.dtype == SERE_F32 ? 4 : 2;
    const size_t T = (size_t)cfg.num_tokens, dh = (size_t)cfg.hidden, M = (size_t)cfg.num_experts;
    const size_t K = (size_t)cfg.top_k, dm = (size_t)cfg.inter, n_sh = (size_t)cfg.num_shared;
    const size_t A = T * K;

    void *hidden = upload(dir, "hidden.bin", T * dh * eb);
    void *router_w = upload(dir, "router_w.bin", M * dh * eb);
    void *w_gate_up = upload(dir, "w_gate_up.bin", M * 2 * dm * dh * eb);
    void *w_down = upload(dir, "w_down.bin", M * dh * dm * eb);
    void *shared_gate_up = n_sh ? upload(dir, "shared_gate_up.bin", n_sh * 2 * dm * dh * eb) : NULL;
    void *shared_down = n_sh ? upload(dir, "shared_down.bin", n_sh * dh * dm * eb) : NULL;
    float *sim = (float *)upload(dir, "sim.bin", M * M * sizeof(float));

    void *out = device_alloc(T * dh * eb);
    void *out_baseline = device_alloc(T * dh * eb);
    void *workspace = device_alloc(ws_bytes);
    sere_route_out r;
    r.topk_ids = (int32_t *)device_alloc(A * 4);
    r.topk_weights = (float *)device_alloc(A * 4);
    r.rerouted_ids = (int32_t *)device_alloc(A * 4);
    r.count_before = (int32_t *)device_alloc(M * 4);
    r.count_after = (int32_t *)device_alloc(M * 4);
    r.primary_mask = (int32_t *)device_alloc(M * 4);
    r.num_active = (int32_t *)device_alloc(2 * 4);
    r.expert_offsets = (int32_t *)device_alloc((M + 1) * 4);
    r.sorted_token = (int32_t *)device_alloc(A * 4);
    r.sorted_slot = (int32_t *)device_alloc(A * 4);

    hipStream_t stream;
    check_hip(hipStreamCreate(&stream), "hipStreamCreate");
    check_sere(sere_moe_decode_baseline(&cfg, hidden, router_w, w_gate_up, w_down, shared_gate_up,
                                        shared_down, out_baseline, NULL, workspace, ws_bytes, stream),
               "sere_moe_decode_baseline");
    check_sere(sere_moe_decode(&cfg, hidden, router_w, w_gate_up, w_down, shared_gate_up, shared_down,
                               sim, out, &r, workspace, ws_bytes, stream),
               "sere_moe_decode");
    check_hip(hipStreamSynchronize(stream), "hipStreamSynchronize");

    download(dir, "out.bin", out, T * dh * eb);
    download(dir, "out_baseline.bin", out_baseline, T * dh * eb);
    download(dir, "topk_ids.bin", r.topk_ids, A * 4);
    download(dir, "topk_weights.bin", r.topk_weights, A * 4);
    download(dir, "rerouted_ids.bin", r.rerouted_ids, A * 4);
    download(dir, "count_before.bin", r.count_before, M * 4);
    download(dir, "count_after.bin", r.count_after, M * 4);
    download(dir, "primary_mask.bin", r.primary_mask, M * 4);
    download(dir, "num_active.bin", r.num_active, 2 * 4);
    download(dir, "expert_offsets.bin", r.expert_offsets, (M + 1) * 4);
    download(dir, "sorted_token.bin", r.sorted_token, A * 4);
    download(dir, "sorted_slot.bin", r.sorted_slot, A * 4);

    int32_t active[2];
    check_hip(hipMemcpy(active, r.num_active, sizeof active, hipMemcpyDeviceToHost), "hipMemcpy to host");
    check_hip(hipStreamDestroy(stream), "hipStreamDestroy");
    for (int i = 0; i < g_num_device; ++i)
        check_hip(hipFree(g_device[i]), "hipFree");
    printf("abi_cli: ok, %d -> %d active experts\n", (int)active[0], (int)active[1]);
    return 0;
}
