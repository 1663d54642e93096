/* A plain C host program that drives the library through its C ABI alone (no Python, no PyTorch):
 * hipMalloc'ed buffers, the calls of include/bitlinear.h, results printed as integers so that the
 * test that runs this program can compare them with the CPU oracle on the same inputs.
 *
 * Inputs come from the 64-bit LCG below (Knuth's MMIX constants); tests/test_gpu_c_abi.py
 * regenerates them.  usage: abi_check N K M
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "bitlinear.h"
#include "bitlinear_decoder.h"

#define HIP(call)                                                                         \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));             \
            return 2;                                                                     \
        }                                                                                 \
    } while (0)
#define BL(call)                                                                          \
    do {                                                                                  \
        bl_status s_ = (call);                                                            \
        if (s_ != BL_OK) {                                                                \
            fprintf(stderr, "%s failed: %s (%s)\n", #call, bl_status_str(s_), bl_last_hip_error()); \
            return 3;                                                                     \
        }                                                                                 \
    } while (0)

static uint64_t lcg_state;
static uint32_t lcg(void) {
    lcg_state = lcg_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (uint32_t)(lcg_state >> 33);
}

static void print_i32(const char *name, const int32_t *v, size_t n) {
    printf("%s", name);
    for (size_t i = 0; i < n; ++i) printf(" %d", v[i]);
    printf("\n");
}
static void print_f32_bits(const char *name, const float *v, size_t n) {
    printf("%s", name);
    for (size_t i = 0; i < n; ++i) {
        uint32_t u;
        memcpy(&u, &v[i], 4);
        printf(" %08x", u);
    }
    printf("\n");
}

int main(int argc, char **argv) {
    if (argc != 4) {
        fprintf(stderr, "usage: %s N K M\n", argv[0]);
        return 1;
    }
    const int64_t N = atoll(argv[1]), K = atoll(argv[2]), M = atoll(argv[3]);
    printf("version %s\n", bl_version());

    /* inputs */
    lcg_state = 20241016u;
    int8_t *w = malloc((size_t)(N * K));
    float *x = malloc((size_t)(M * K) * sizeof(float));
    for (int64_t i = 0; i < N * K; ++i) w[i] = (int8_t)(lcg() % 3) - 1;
    for (int64_t i = 0; i < M * K; ++i) x[i] = (float)((int)(lcg() % 2001) - 1000) / 256.0f;
    const float w_scale = 0.03125f;

    bl_packed_desc d;
    BL(bl_packed_desc_init(N, K, w_scale, &d));
    const int64_t Kp = bl_padded_k(K);
    printf("desc %lld %lld %lld %lld %llu\n", (long long)d.N, (long long)d.K, (long long)d.Np, (long long)d.Kp,
           (unsigned long long)d.bytes);

    int8_t *w_dev, *w_back_dev, *q_dev;
    void *packed_dev, *x_dev, *ws_dev;
    float *a_scale_dev, *out_dev, *out2_dev;
    int32_t *q_sum_dev, *acc_dev, *acc2_dev, *bad_dev;
    HIP(hipMalloc((void **)&w_dev, (size_t)(N * K)));
    HIP(hipMalloc((void **)&w_back_dev, (size_t)(N * K)));
    HIP(hipMalloc(&packed_dev, d.bytes));
    HIP(hipMalloc(&x_dev, (size_t)(M * K) * 4));
    HIP(hipMalloc((void **)&q_dev, (size_t)(M * Kp)));
    HIP(hipMalloc((void **)&a_scale_dev, (size_t)M * 4));
    HIP(hipMalloc((void **)&q_sum_dev, (size_t)M * 4));
    HIP(hipMalloc((void **)&out_dev, (size_t)(M * N) * 4));
    HIP(hipMalloc((void **)&out2_dev, (size_t)(M * N) * 4));
    HIP(hipMalloc((void **)&acc_dev, (size_t)(M * N) * 4));
    HIP(hipMalloc((void **)&acc2_dev, (size_t)(M * N) * 4));
    HIP(hipMalloc((void **)&bad_dev, 4));
    HIP(hipMalloc(&ws_dev, BL_WORKSPACE_BYTES));
    HIP(hipMemset(ws_dev, 0, BL_WORKSPACE_BYTES));
    HIP(hipMemset(bad_dev, 0, 4));
    HIP(hipMemcpy(w_dev, w, (size_t)(N * K), hipMemcpyHostToDevice));
    HIP(hipMemcpy(x_dev, x, (size_t)(M * K) * 4, hipMemcpyHostToDevice));

    /* pack, unpack, round trip */
    BL(bl_pack_ternary(w_dev, &d, packed_dev, bad_dev, NULL));
    BL(bl_unpack_ternary(packed_dev, &d, w_back_dev, NULL));
    int8_t *w_back = malloc((size_t)(N * K));
    int32_t bad = -1;
    HIP(hipMemcpy(w_back, w_back_dev, (size_t)(N * K), hipMemcpyDeviceToHost));
    HIP(hipMemcpy(&bad, bad_dev, 4, hipMemcpyDeviceToHost));
    printf("roundtrip %d bad %d\n", memcmp(w, w_back, (size_t)(N * K)) == 0, bad);

    /* quantize, decode product, prefill product */
    BL(bl_quant_act(x_dev, BL_F32, M, K, K, q_dev, a_scale_dev, q_sum_dev, NULL));
    BL(bl_gemv(packed_dev, &d, q_dev, a_scale_dev, q_sum_dev, M, out_dev, acc_dev, NULL));
    BL(bl_gemm(packed_dev, &d, q_dev, a_scale_dev, q_sum_dev, M, out2_dev, acc2_dev, NULL));
    HIP(hipDeviceSynchronize());
    int8_t *q = malloc((size_t)(M * Kp));
    float *a_scale = malloc((size_t)M * 4), *out = malloc((size_t)(M * N) * 4), *out2 = malloc((size_t)(M * N) * 4);
    int32_t *q_sum = malloc((size_t)M * 4), *acc = malloc((size_t)(M * N) * 4), *acc2 = malloc((size_t)(M * N) * 4);
    HIP(hipMemcpy(q, q_dev, (size_t)(M * Kp), hipMemcpyDeviceToHost));
    HIP(hipMemcpy(a_scale, a_scale_dev, (size_t)M * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(q_sum, q_sum_dev, (size_t)M * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(out, out_dev, (size_t)(M * N) * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(acc, acc_dev, (size_t)(M * N) * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(out2, out2_dev, (size_t)(M * N) * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(acc2, acc2_dev, (size_t)(M * N) * 4, hipMemcpyDeviceToHost));
    printf("q");
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < Kp; ++k) printf(" %d", q[m * Kp + k]);
    printf("\n");
    print_f32_bits("a_scale", a_scale, (size_t)M);
    print_i32("q_sum", q_sum, (size_t)M);
    print_i32("acc_gemv", acc, (size_t)(M * N));
    print_f32_bits("out_gemv", out, (size_t)(M * N));
    printf("gemm_equals_gemv %d %d\n", memcmp(acc, acc2, (size_t)(M * N) * 4) == 0, memcmp(out, out2, (size_t)(M * N) * 4) == 0);

    /* fused decode launch of two problems sharing the input's first row, with the workspace */
    bl_decode_item items[2];
    memset(items, 0, sizeof items);
    for (int i = 0; i < 2; ++i) {
        items[i].x_dev = x_dev;
        items[i].dt = BL_F32;
        items[i].ldx = K;
        items[i].packed_dev = packed_dev;
        items[i].desc = &d;
        items[i].out_dev = i ? out2_dev : out_dev;
        items[i].acc_dev = i ? acc2_dev : acc_dev;
    }
    HIP(hipMemset(acc_dev, 0xff, (size_t)N * 4));
    HIP(hipMemset(acc2_dev, 0xff, (size_t)N * 4));
    BL(bl_decode_batch(items, 2, 1, ws_dev, NULL));
    HIP(hipDeviceSynchronize());
    HIP(hipMemcpy(acc, acc_dev, (size_t)N * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(acc2, acc2_dev, (size_t)N * 4, hipMemcpyDeviceToHost));
    print_i32("acc_fused", acc, (size_t)N);
    printf("fused_pair_equal %d\n", memcmp(acc, acc2, (size_t)N * 4) == 0);

    /* the 1.78-bit layout: round trip, and the one-token product equals the 2-bit one on the same weights */
    {
        bl_packed_desc d2;
        BL(bl_tl2_desc_init(N, K, w_scale, &d2));
        const int64_t q_bytes = bl_tl2_padded_k(K) > Kp ? bl_tl2_padded_k(K) : Kp;
        void *packed2_dev;
        int8_t *q2_dev;
        HIP(hipMalloc(&packed2_dev, d2.bytes));
        HIP(hipMalloc((void **)&q2_dev, (size_t)q_bytes));
        HIP(hipMemset(q2_dev, 0, (size_t)q_bytes));
        HIP(hipMemset(w_back_dev, 9, (size_t)(N * K)));
        BL(bl_tl2_pack(w_dev, &d2, packed2_dev, bad_dev, NULL));
        BL(bl_tl2_unpack(packed2_dev, &d2, w_back_dev, NULL));
        BL(bl_quant_act(x_dev, BL_F32, 1, K, K, q2_dev, a_scale_dev, q_sum_dev, NULL));
        BL(bl_tl2_gemv(packed2_dev, &d2, q2_dev, a_scale_dev, out_dev, acc_dev, NULL));
        BL(bl_gemv(packed_dev, &d, q2_dev, a_scale_dev, q_sum_dev, 1, out2_dev, acc2_dev, NULL));
        HIP(hipDeviceSynchronize());
        HIP(hipMemcpy(w_back, w_back_dev, (size_t)(N * K), hipMemcpyDeviceToHost));
        HIP(hipMemcpy(acc, acc_dev, (size_t)N * 4, hipMemcpyDeviceToHost));
        HIP(hipMemcpy(acc2, acc2_dev, (size_t)N * 4, hipMemcpyDeviceToHost));
        HIP(hipMemcpy(out, out_dev, (size_t)N * 4, hipMemcpyDeviceToHost));
        HIP(hipMemcpy(out2, out2_dev, (size_t)N * 4, hipMemcpyDeviceToHost));
        printf("tl2_desc %lld %llu\n", (long long)d2.Kp, (unsigned long long)d2.bytes);
        printf("tl2_roundtrip %d\n", memcmp(w, w_back, (size_t)(N * K)) == 0);
        print_i32("acc_tl2", acc, (size_t)N);
        printf("tl2_equals_gemv %d %d\n", memcmp(acc, acc2, (size_t)N * 4) == 0, memcmp(out, out2, (size_t)N * 4) == 0);
    }

    /* the decoder block's norm: stand-alone (norm + quantizer) and folded into the product (K % 8 == 0) */
    {
        float *gamma = malloc((size_t)K * 4), *gamma_dev, *y_dev, *h_out_dev;
        for (int64_t k = 0; k < K; ++k) gamma[k] = 0.5f + (float)(lcg() % 1024) / 1024.0f;
        HIP(hipMalloc((void **)&gamma_dev, (size_t)K * 4));
        HIP(hipMalloc((void **)&y_dev, (size_t)K * 4));
        HIP(hipMalloc((void **)&h_out_dev, (size_t)K * 4));
        HIP(hipMemcpy(gamma_dev, gamma, (size_t)K * 4, hipMemcpyHostToDevice));
        bl_norm_quant_args na;
        memset(&na, 0, sizeof na);
        na.mode = BL_NORM_PLAIN;
        na.M = 1;
        na.K = K;
        na.Kp = Kp;
        na.a_dev = (const float *)x_dev;
        na.gamma_dev = gamma_dev;
        na.eps = 1e-5f;
        na.q_dev = q_dev;
        na.a_scale_dev = a_scale_dev;
        na.q_sum_dev = q_sum_dev;
        na.y_dev = y_dev;
        BL(bl_norm_quant(&na, NULL));
        HIP(hipDeviceSynchronize());
        float *y = malloc((size_t)K * 4);
        HIP(hipMemcpy(y, y_dev, (size_t)K * 4, hipMemcpyDeviceToHost));
        HIP(hipMemcpy(q, q_dev, (size_t)Kp, hipMemcpyDeviceToHost));
        HIP(hipMemcpy(a_scale, a_scale_dev, 4, hipMemcpyDeviceToHost));
        HIP(hipMemcpy(q_sum, q_sum_dev, 4, hipMemcpyDeviceToHost));
        print_f32_bits("norm_y", y, (size_t)K);
        printf("norm_q");
        for (int64_t k = 0; k < Kp; ++k) printf(" %d", q[k]);
        printf("\n");
        print_f32_bits("norm_a_scale", a_scale, 1);
        print_i32("norm_q_sum", q_sum, 1);
        if (K % 8 == 0) {
            bl_decode_norm_item ni;
            memset(&ni, 0, sizeof ni);
            ni.x_dev = (const float *)x_dev;
            ni.delta_dev = (const float *)x_dev;   /* x' = 2 x */
            ni.h_out_dev = h_out_dev;
            ni.gamma_dev = gamma_dev;
            ni.eps = 1e-5f;
            ni.packed_dev = packed_dev;
            ni.desc = &d;
            ni.out_dev = out_dev;
            ni.acc_dev = acc_dev;
            ni.a_scale_dev = a_scale_dev;
            BL(bl_decode_norm_batch(&ni, 1, ws_dev, NULL));
            HIP(hipDeviceSynchronize());
            HIP(hipMemcpy(acc, acc_dev, (size_t)N * 4, hipMemcpyDeviceToHost));
            HIP(hipMemcpy(out, out_dev, (size_t)N * 4, hipMemcpyDeviceToHost));
            HIP(hipMemcpy(a_scale, a_scale_dev, 4, hipMemcpyDeviceToHost));
            HIP(hipMemcpy(y, h_out_dev, (size_t)K * 4, hipMemcpyDeviceToHost));
            print_i32("fold_acc", acc, (size_t)N);
            print_f32_bits("fold_out", out, (size_t)N);
            print_f32_bits("fold_a_scale", a_scale, 1);
            print_f32_bits("fold_h", y, (size_t)K);
        }
        printf("err_norm_null %d\n", (int)bl_norm_quant(NULL, NULL));
    }

    /* argument errors come back as codes, before anything is launched */
    printf("err_m_range %d\n", (int)bl_gemv(packed_dev, &d, q_dev, a_scale_dev, q_sum_dev, 9, out_dev, NULL, NULL));
    printf("err_null %d\n", (int)bl_gemv(NULL, &d, q_dev, a_scale_dev, q_sum_dev, 1, out_dev, NULL, NULL));
    printf("done\n");
    return 0;
}
