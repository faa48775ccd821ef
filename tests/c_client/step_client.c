/* A client of the C ABI with no Python and no PyTorch in the process: plain C99, device memory from hipMalloc.
 *
 *   step_client <input file> <output file>
 *
 * The input file (written by tests/test_gpu_c_client.py, native endianness) holds
 *   int32  L, R, pack_align
 *   L x { int64 elem_off; int32 c_out, c_in, khw, mode, k, k_in }
 *   int64  arena_elems
 *   R x arena_elems float   the replicas
 *   arena_elems float       the dual U
 * The program runs one outer step -- hsadmm_project_compact, hsadmm_expand -- then the same step again from the
 * first step's dual and selection record through hsadmm_step with a prediction and the dual out of place, and writes
 * for each of the two steps: Z, the new dual, dst (arena_elems floats each), mask (groups_total bytes),
 * layer_off (L + 1 int64), then packed (layer_off[L] floats).
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "hsadmm.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_HS(x) do { int rc_ = (x); if (rc_ != HSADMM_OK) { \
    fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hsadmm_strerror(rc_)); return 3; } } while (0)

static int read_all(FILE* f, void* p, size_t bytes) { return fread(p, 1, bytes, f) == bytes ? 0 : -1; }

static int dump(FILE* f, const void* dev, size_t bytes)
{
    void* h = malloc(bytes ? bytes : 1);
    if (!h) return -1;
    if (hipMemcpy(h, dev, bytes, hipMemcpyDeviceToHost) != hipSuccess) { free(h); return -1; }
    const int ok = fwrite(h, 1, bytes, f) == bytes ? 0 : -1;
    free(h);
    return ok;
}

int main(int argc, char** argv)
{
    if (argc != 3) { fprintf(stderr, "usage: %s <input> <output>\n", argv[0]); return 1; }
    FILE* in = fopen(argv[1], "rb");
    if (!in) { perror(argv[1]); return 1; }
    int32_t hdr[3];
    if (read_all(in, hdr, sizeof hdr)) return 1;
    const int32_t L = hdr[0], R = hdr[1], pack_align = hdr[2];
    if (L < 1 || R < 1 || R > HSADMM_MAX_REPLICAS) return 1;
    hsadmm_layer_t* layers = (hsadmm_layer_t*)calloc((size_t)L, sizeof *layers);
    if (!layers) return 1;
    for (int32_t l = 0; l < L; ++l) {
        int64_t off;
        int32_t f[6];
        if (read_all(in, &off, sizeof off) || read_all(in, f, sizeof f)) return 1;
        layers[l].elem_off = off;
        layers[l].c_out = f[0]; layers[l].c_in = f[1]; layers[l].khw = f[2];
        layers[l].mode = f[3]; layers[l].k = f[4]; layers[l].k_in = f[5];
    }
    int64_t n = 0;
    if (read_all(in, &n, sizeof n) || n < 1) return 1;
    const size_t ab = (size_t)n * sizeof(float);
    float* host = (float*)malloc(ab);
    if (!host) return 1;

    CHECK_HIP(hipSetDevice(0));
    hsadmm_plan_t* plan = NULL;
    CHECK_HS(hsadmm_plan_create(layers, L, pack_align, &plan));
    int64_t arena = 0, groups = 0, cap = 0;
    size_t ws_bytes = 0;
    CHECK_HS(hsadmm_plan_sizes(plan, &arena, &groups, &cap, &ws_bytes));
    if (arena != n) { fprintf(stderr, "arena size %lld, file says %lld\n", (long long)arena, (long long)n); return 1; }

    const float* W[HSADMM_MAX_REPLICAS];
    float* dW[HSADMM_MAX_REPLICAS];
    for (int32_t r = 0; r < R; ++r) {
        if (read_all(in, host, ab)) return 1;
        CHECK_HIP(hipMalloc((void**)&dW[r], ab));
        CHECK_HIP(hipMemcpy(dW[r], host, ab, hipMemcpyHostToDevice));
        W[r] = dW[r];
    }
    float *U, *U2, *Z, *dst, *packed;
    uint8_t* mask;
    int64_t* off;
    int32_t *kept, *sel0, *sel1;
    void* ws;
    if (read_all(in, host, ab)) return 1;
    fclose(in);
    CHECK_HIP(hipMalloc((void**)&U, ab));
    CHECK_HIP(hipMemcpy(U, host, ab, hipMemcpyHostToDevice));
    CHECK_HIP(hipMalloc((void**)&U2, ab));
    CHECK_HIP(hipMemset(U2, 0xff, ab));
    CHECK_HIP(hipMalloc((void**)&Z, ab));
    CHECK_HIP(hipMalloc((void**)&dst, ab));
    CHECK_HIP(hipMalloc((void**)&packed, (size_t)(cap > 0 ? cap : 1) * sizeof(float)));
    CHECK_HIP(hipMalloc((void**)&mask, (size_t)groups));
    CHECK_HIP(hipMalloc((void**)&off, (size_t)(L + 1) * sizeof(int64_t)));
    CHECK_HIP(hipMalloc((void**)&kept, (size_t)groups * sizeof(int32_t)));
    CHECK_HIP(hipMalloc((void**)&sel0, (size_t)groups * sizeof(int32_t)));
    CHECK_HIP(hipMalloc((void**)&sel1, (size_t)groups * sizeof(int32_t)));
    CHECK_HIP(hipMalloc(&ws, ws_bytes));
    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));

    FILE* out = fopen(argv[2], "wb");
    if (!out) { perror(argv[2]); return 1; }
    int64_t* off_h = (int64_t*)malloc((size_t)(L + 1) * sizeof(int64_t));
    if (!off_h) return 1;

    /* step 1: the named calls; the selection record for the next step comes from the mask */
    CHECK_HS(hsadmm_project_compact(plan, W, R, U, Z, NULL, mask, NULL, packed, off, kept, ws, ws_bytes, stream));
    CHECK_HS(hsadmm_expand(plan, packed, NULL, dst, ws, ws_bytes, stream));
    CHECK_HS(hsadmm_selection_from_mask(plan, mask, sel0, ws, ws_bytes, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_HIP(hipMemcpy(off_h, off, (size_t)(L + 1) * sizeof(int64_t), hipMemcpyDeviceToHost));
    if (dump(out, Z, ab) || dump(out, U, ab) || dump(out, dst, ab) || dump(out, mask, (size_t)groups) ||
        dump(out, off, (size_t)(L + 1) * sizeof(int64_t)) || dump(out, packed, (size_t)off_h[L] * sizeof(float)))
        return 4;

    /* step 2: the one entry point, predicted by step 1's selection, the dual written to a second buffer */
    hsadmm_step_args_t a;
    memset(&a, 0, sizeof a);
    a.struct_bytes = sizeof a;
    a.W_replicas = W; a.R = R;
    a.U = U; a.U_out = U2; a.Z = Z; a.mask = mask;
    a.sel_prev = sel0; a.sel = sel1;
    a.packed = packed; a.layer_off = off; a.kept_idx = kept;
    a.workspace = ws; a.workspace_bytes = ws_bytes; a.hip_stream = stream;
    CHECK_HS(hsadmm_step(plan, &a));
    CHECK_HS(hsadmm_expand(plan, packed, NULL, dst, ws, ws_bytes, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_HIP(hipMemcpy(off_h, off, (size_t)(L + 1) * sizeof(int64_t), hipMemcpyDeviceToHost));
    if (dump(out, Z, ab) || dump(out, U2, ab) || dump(out, dst, ab) || dump(out, mask, (size_t)groups) ||
        dump(out, off, (size_t)(L + 1) * sizeof(int64_t)) || dump(out, packed, (size_t)off_h[L] * sizeof(float)))
        return 4;
    fclose(out);

    hsadmm_plan_destroy(plan);
    for (int32_t r = 0; r < R; ++r) (void)hipFree(dW[r]);
    (void)hipFree(U); (void)hipFree(U2); (void)hipFree(Z); (void)hipFree(dst); (void)hipFree(packed);
    (void)hipFree(mask); (void)hipFree(off); (void)hipFree(kept); (void)hipFree(sel0); (void)hipFree(sel1);
    (void)hipFree(ws);
    (void)hipStreamDestroy(stream);
    free(host); free(off_h); free(layers);
    printf("step_client: ok\n");
    return 0;
}
