// C-ABI entry points: host-side validation, then one kernel launch each.
// No entry point allocates, frees or synchronizes.
#include <stdio.h>
#include <string.h>

#include "bl_internal.hpp"

namespace {

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

bl_status check_desc(const bl_packed_desc* d) {
    if (!d) return BL_ERR_NULL;
    if (d->version != BL_LAYOUT_VERSION) return BL_ERR_LAYOUT;
    if (d->N < 1 || d->K < 1 || d->K > BL_MAX_K || d->N > INT32_MAX - BL_TILE_N) return BL_ERR_SHAPE;
    if (d->Np != bl_padded_n(d->N) || d->Kp != bl_padded_k(d->K)) return BL_ERR_SHAPE;
    if (d->bytes != (uint64_t)d->Np * (uint64_t)d->Kp / 4) return BL_ERR_BUF_SMALL;
    return BL_OK;
}

bl_status check_product_args(const void* packed, const bl_packed_desc* d, const int8_t* q, const float* a_scale,
                             const int32_t* q_sum, int64_t M, const float* out, const int32_t* acc) {
    if (!packed || !d || !q || !a_scale || !q_sum || !out) return BL_ERR_NULL;
    bl_status s = check_desc(d);
    if (s != BL_OK) return s;
    if (M < 1 || M > INT32_MAX / 2) return BL_ERR_SHAPE;
    if (!aligned(packed, 16) || !aligned(q, 16) || !aligned(a_scale, 4) || !aligned(q_sum, 4) ||
        !aligned(out, 4) || (acc && !aligned(acc, 4)))
        return BL_ERR_ALIGN;
    return BL_OK;
}

bl_status check_tl2_desc(const bl_packed_desc* d) {
    if (!d) return BL_ERR_NULL;
    if (d->version != BL_TL2_LAYOUT_VERSION) return BL_ERR_LAYOUT;
    if (d->N < 1 || d->K < 1 || d->K > BL_MAX_K || d->N > INT32_MAX - BL_TILE_N) return BL_ERR_SHAPE;
    if (d->Np != bl_padded_n(d->N) || d->Kp != bl_tl2_padded_k(d->K)) return BL_ERR_SHAPE;
    if (d->bytes != (uint64_t)d->Np * (uint64_t)(d->Kp / BL_TL2_TILE_K) * 16) return BL_ERR_BUF_SMALL;
    return BL_OK;
}

bl::GemmProblem make_problem(const void* packed, const bl_packed_desc* d, const int8_t* q, const float* a_scale,
                             const int32_t* q_sum, float* out, int32_t* acc) {
    bl::GemmProblem p;
    p.packed = static_cast<const uint4*>(packed);
    p.q = reinterpret_cast<const int32_t*>(q);
    p.a_scale = a_scale;
    p.q_sum = q_sum;
    p.out = out;
    p.acc = acc;
    p.N = (int32_t)d->N;
    p.KC = (int32_t)(d->Kp / BL_TILE_K);
    p.row_blocks = (int32_t)(d->Np / BL_TILE_N);
    p.w_scale = d->w_scale;
    return p;
}

thread_local hipError_t t_last_hip_error = hipSuccess;
thread_local char t_kernel_text[160];

inline bl_status hip_status(hipError_t e) {
    t_last_hip_error = e;
    return e == hipSuccess ? BL_OK : BL_ERR_HIP;
}

// hipGetLastError() reports the most recent error of ANY earlier HIP call on this thread, also
// other libraries' (benign, already handled) ones.  Drop those so that the check after our launch
// sees only our launch.
inline void drop_stale_hip_error() { (void)hipGetLastError(); }

}  // namespace

thread_local bl::KernelNote bl::t_kernel_note;

extern "C" {

int64_t bl_padded_k(int64_t K) {
    if (K < 1 || K > BL_MAX_K) return -1;
    return (K + BL_TILE_K - 1) / BL_TILE_K * BL_TILE_K;
}

int64_t bl_padded_n(int64_t N) {
    if (N < 1 || N > INT32_MAX - BL_TILE_N) return -1;
    return (N + BL_TILE_N - 1) / BL_TILE_N * BL_TILE_N;
}

bl_status bl_packed_desc_init(int64_t N, int64_t K, float w_scale, bl_packed_desc* d) {
    if (!d) return BL_ERR_NULL;
    if (bl_padded_n(N) < 0 || bl_padded_k(K) < 0) return BL_ERR_SHAPE;
    memset(d, 0, sizeof *d);
    d->version = BL_LAYOUT_VERSION;
    d->N = N;
    d->K = K;
    d->Np = bl_padded_n(N);
    d->Kp = bl_padded_k(K);
    d->bytes = (uint64_t)d->Np * (uint64_t)d->Kp / 4;
    d->w_scale = w_scale;
    return BL_OK;
}

bl_status bl_pack_ternary(const int8_t* w_dev, const bl_packed_desc* d, void* packed_dev, int32_t* bad_count_dev,
                          void* stream) {
    if (!w_dev || !d || !packed_dev) return BL_ERR_NULL;
    bl_status s = check_desc(d);
    if (s != BL_OK) return s;
    if (!aligned(packed_dev, 16) || (bad_count_dev && !aligned(bad_count_dev, 4))) return BL_ERR_ALIGN;
    drop_stale_hip_error();
    return hip_status(bl::launch_pack(w_dev, nullptr, d->N, d->K, d->Np, d->Kp, static_cast<uint32_t*>(packed_dev),
                                      bad_count_dev, static_cast<hipStream_t>(stream)));
}

bl_status bl_pack_gate_up(const int8_t* gate_dev, const int8_t* up_dev, const bl_packed_desc* d, void* packed_dev,
                          int32_t* bad_count_dev, void* stream) {
    if (!gate_dev || !up_dev || !d || !packed_dev) return BL_ERR_NULL;
    bl_status s = check_desc(d);
    if (s != BL_OK) return s;
    if (d->N % BL_TILE_N != 0) return BL_ERR_SHAPE;   // 2 F rows, F a multiple of 32
    if (!aligned(packed_dev, 16) || (bad_count_dev && !aligned(bad_count_dev, 4))) return BL_ERR_ALIGN;
    drop_stale_hip_error();
    return hip_status(bl::launch_pack(gate_dev, up_dev, d->N, d->K, d->Np, d->Kp, static_cast<uint32_t*>(packed_dev),
                                      bad_count_dev, static_cast<hipStream_t>(stream)));
}

bl_status bl_unpack_ternary(const void* packed_dev, const bl_packed_desc* d, int8_t* w_dev, void* stream) {
    if (!w_dev || !d || !packed_dev) return BL_ERR_NULL;
    bl_status s = check_desc(d);
    if (s != BL_OK) return s;
    if (!aligned(packed_dev, 16)) return BL_ERR_ALIGN;
    drop_stale_hip_error();
    return hip_status(bl::launch_unpack(static_cast<const uint32_t*>(packed_dev), d->N, d->K, d->Np, d->Kp, w_dev,
                                        static_cast<hipStream_t>(stream)));
}

int64_t bl_tl2_padded_k(int64_t K) {
    if (K < 1 || K > BL_MAX_K) return -1;
    return (K + BL_TL2_TILE_K - 1) / BL_TL2_TILE_K * BL_TL2_TILE_K;
}

bl_status bl_tl2_desc_init(int64_t N, int64_t K, float w_scale, bl_packed_desc* d) {
    if (!d) return BL_ERR_NULL;
    if (bl_padded_n(N) < 0 || bl_tl2_padded_k(K) < 0) return BL_ERR_SHAPE;
    memset(d, 0, sizeof *d);
    d->version = BL_TL2_LAYOUT_VERSION;
    d->N = N;
    d->K = K;
    d->Np = bl_padded_n(N);
    d->Kp = bl_tl2_padded_k(K);
    d->bytes = (uint64_t)d->Np * (uint64_t)(d->Kp / BL_TL2_TILE_K) * 16;
    d->w_scale = w_scale;
    return BL_OK;
}

bl_status bl_tl2_pack(const int8_t* w_dev, const bl_packed_desc* d, void* packed_dev, int32_t* bad_count_dev,
                      void* stream) {
    if (!w_dev || !d || !packed_dev) return BL_ERR_NULL;
    bl_status s = check_tl2_desc(d);
    if (s != BL_OK) return s;
    if (!aligned(packed_dev, 16) || (bad_count_dev && !aligned(bad_count_dev, 4))) return BL_ERR_ALIGN;
    drop_stale_hip_error();
    return hip_status(bl::launch_tl2_pack(w_dev, d->N, d->K, d->Np, d->Kp, static_cast<uint32_t*>(packed_dev),
                                          bad_count_dev, static_cast<hipStream_t>(stream)));
}

bl_status bl_tl2_unpack(const void* packed_dev, const bl_packed_desc* d, int8_t* w_dev, void* stream) {
    if (!w_dev || !d || !packed_dev) return BL_ERR_NULL;
    bl_status s = check_tl2_desc(d);
    if (s != BL_OK) return s;
    if (!aligned(packed_dev, 16)) return BL_ERR_ALIGN;
    drop_stale_hip_error();
    return hip_status(bl::launch_tl2_unpack(static_cast<const uint32_t*>(packed_dev), d->N, d->K, d->Np, d->Kp,
                                            w_dev, static_cast<hipStream_t>(stream)));
}

bl_status bl_tl2_gemv_batch(const bl_gemv_item* items, int32_t count, void* workspace_dev, void* stream) {
    if (!items) return BL_ERR_NULL;
    if (count < 1 || count > BL_MAX_BATCH) return BL_ERR_COUNT;
    if (workspace_dev && !aligned(workspace_dev, 256)) return BL_ERR_ALIGN;
    bl::DecodeBatch b;
    memset(&b, 0, sizeof b);
    b.ws = static_cast<unsigned long long*>(workspace_dev);
    b.layout = 2;
    for (int i = 0; i < count; ++i) {
        const bl_gemv_item& it = items[i];
        if (!it.packed_dev || !it.desc || !it.q_dev || !it.a_scale_dev || !it.out_dev) return BL_ERR_NULL;
        bl_status s = check_tl2_desc(it.desc);
        if (s != BL_OK) return s;
        if (!aligned(it.packed_dev, 16) || !aligned(it.q_dev, 16) || !aligned(it.a_scale_dev, 4) ||
            !aligned(it.out_dev, 4) || (it.acc_dev && !aligned(it.acc_dev, 4)))
            return BL_ERR_ALIGN;
        bl::DecodeProblem& p = b.p[i];
        p.packed = static_cast<const uint4*>(it.packed_dev);
        p.q = reinterpret_cast<const int32_t*>(it.q_dev);
        p.a_scale = it.a_scale_dev;
        p.out = it.out_dev;
        p.acc = it.acc_dev;
        p.N = (int32_t)it.desc->N;
        p.K = (int32_t)it.desc->K;
        p.KC = (int32_t)(it.desc->Kp / BL_TL2_TILE_K);
        p.row_blocks = (int32_t)(it.desc->Np / BL_TILE_N);
        p.w_scale = it.desc->w_scale;
    }
    b.count = count;
    drop_stale_hip_error();
    return hip_status(bl::launch_decode(b, 1, false, static_cast<hipStream_t>(stream)));
}

bl_status bl_tl2_gemv(const void* packed_dev, const bl_packed_desc* d, const int8_t* q_dev, const float* a_scale_dev,
                      float* out_dev, int32_t* acc_dev, void* stream) {
    const bl_gemv_item it = {packed_dev, d, q_dev, a_scale_dev, nullptr, out_dev, acc_dev};
    return bl_tl2_gemv_batch(&it, 1, nullptr, stream);
}

static bl_status fill_quant_problem(const bl_quant_item& it, bl::QuantProblem& p) {
    if (!it.x_dev || !it.q_dev || !it.a_scale_dev) return BL_ERR_NULL;
    if (it.dt != BL_F32 && it.dt != BL_BF16) return BL_ERR_DTYPE;
    const int64_t Kp = bl_padded_k(it.K);
    if (it.M < 1 || it.M > INT32_MAX / 2 || Kp < 0 || it.ldx < it.K) return BL_ERR_SHAPE;
    if (!aligned(it.x_dev, it.dt == BL_F32 ? 4 : 2) || !aligned(it.q_dev, 16) || !aligned(it.a_scale_dev, 4) ||
        (it.q_sum_dev && !aligned(it.q_sum_dev, 4)))
        return BL_ERR_ALIGN;
    const bool vec = (it.K % 8 == 0) && (it.ldx % 8 == 0) && aligned(it.x_dev, 16);
    p.x = it.x_dev;
    p.q = it.q_dev;
    p.a_scale = it.a_scale_dev;
    p.q_sum = it.q_sum_dev;
    p.ldx = it.ldx;
    p.M = (int32_t)it.M;
    p.K = (int32_t)it.K;
    p.Kp = (int32_t)Kp;
    p.flags = (it.dt == BL_BF16 ? 1 : 0) | (vec ? 2 : 0);
    p.first_row = 0;
    return BL_OK;
}

bl_status bl_quant_act_batch(const bl_quant_item* items, int32_t count, void* stream) {
    if (!items) return BL_ERR_NULL;
    if (count < 1 || count > BL_MAX_BATCH) return BL_ERR_COUNT;
    bl::QuantBatch b;
    memset(&b, 0, sizeof b);
    for (int i = 0; i < count; ++i) {
        bl_status s = fill_quant_problem(items[i], b.p[i]);
        if (s != BL_OK) return s;
    }
    b.count = count;
    drop_stale_hip_error();
    return hip_status(bl::launch_quant(b, static_cast<hipStream_t>(stream)));
}

bl_status bl_quant_act(const void* x_dev, bl_dtype dt, int64_t M, int64_t K, int64_t ldx, int8_t* q_dev,
                       float* a_scale_dev, int32_t* q_sum_dev, void* stream) {
    const bl_quant_item it = {x_dev, dt, M, K, ldx, q_dev, a_scale_dev, q_sum_dev};
    return bl_quant_act_batch(&it, 1, stream);
}

bl_status bl_gemv(const void* packed_dev, const bl_packed_desc* d, const int8_t* q_dev, const float* a_scale_dev,
                  const int32_t* q_sum_dev, int64_t M, float* out_dev, int32_t* acc_dev, void* stream) {
    bl_gemv_item it = {packed_dev, d, q_dev, a_scale_dev, q_sum_dev, out_dev, acc_dev};
    return bl_gemv_batch(&it, 1, M, nullptr, stream);
}

static bl::DecodeProblem make_decode_problem(const void* packed, const bl_packed_desc* d, float* out, int32_t* acc) {
    bl::DecodeProblem p;
    memset(&p, 0, sizeof p);
    p.packed = static_cast<const uint4*>(packed);
    p.out = out;
    p.acc = acc;
    p.N = (int32_t)d->N;
    p.K = (int32_t)d->K;
    p.KC = (int32_t)(d->Kp / BL_TILE_K);
    p.row_blocks = (int32_t)(d->Np / BL_TILE_N);
    p.w_scale = d->w_scale;
    return p;
}

// Validation and problem set-up shared by bl_gemv_batch and bl_gemv_batch_static (no HIP call).
static bl_status fill_gemv_batch(const bl_gemv_item* items, int32_t count, int64_t M, bl::DecodeBatch& b) {
    if (!items) return BL_ERR_NULL;
    if (count < 1 || count > BL_MAX_BATCH) return BL_ERR_COUNT;
    if (M < 1 || M > BL_MAX_GEMV_M) return BL_ERR_M_RANGE;
    memset(&b, 0, sizeof b);
    for (int i = 0; i < count; ++i) {
        const bl_gemv_item& it = items[i];
        bl_status s = check_product_args(it.packed_dev, it.desc, it.q_dev, it.a_scale_dev, it.q_sum_dev, M,
                                         it.out_dev, it.acc_dev);
        if (s != BL_OK) return s;
        b.p[i] = make_decode_problem(it.packed_dev, it.desc, it.out_dev, it.acc_dev);
        b.p[i].q = reinterpret_cast<const int32_t*>(it.q_dev);
        b.p[i].a_scale = it.a_scale_dev;
        b.p[i].q_sum = it.q_sum_dev;
    }
    b.count = count;
    return BL_OK;
}

bl_status bl_gemv_batch(const bl_gemv_item* items, int32_t count, int64_t M, void* workspace_dev, void* stream) {
    bl::DecodeBatch b;
    const bl_status st = fill_gemv_batch(items, count, M, b);
    if (st != BL_OK) return st;
    if (workspace_dev && !aligned(workspace_dev, 256)) return BL_ERR_ALIGN;
    b.ws = static_cast<unsigned long long*>(workspace_dev);
    drop_stale_hip_error();
    return hip_status(bl::launch_decode(b, (int)M, false, static_cast<hipStream_t>(stream)));
}

}  // extern "C"

// ---- bl_gemv_batch_static: the workspace of the work-balanced launch in a static device array -----------------
namespace {

// Each GPU the library runs on holds its own copy of this array, at its own address, until the process ends.  In
// host code the NAME is only a stand-in for hipGetSymbolAddress: kernels, fills and copies take the per-device
// pointer looked up below, never the name.
__device__ __align__(256) unsigned long long scratch[BL_STATIC_WS_WGS * BL_TILE_N];

constexpr int kMaxScratchDevices = 64;
unsigned long long* g_scratch_ptr[kMaxScratchDevices];   // per device ordinal; null until that device's first call

__global__ void scratch_clear_kernel(unsigned long long* ws, int words) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) ws[i] = 0ull;
}

// The current device's copy of `scratch`; on a device's first call its address is looked up and the array is
// cleared by a small kernel on `s` (a fill kernel, not a memset node: the caller's stream may be under capture).
hipError_t scratch_for_current_device(hipStream_t s, unsigned long long** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxScratchDevices) return hipErrorInvalidDevice;
    unsigned long long* ptr = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!ptr) {
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        constexpr int words = BL_STATIC_WS_WGS * BL_TILE_N;
        scratch_clear_kernel<<<dim3((words + 255) / 256), dim3(256), 0, s>>>(ptr, words);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        __atomic_store_n(&g_scratch_ptr[dev], ptr, __ATOMIC_RELEASE);
    }
    *out = ptr;
    return hipSuccess;
}

}  // namespace

extern "C" {

bl_status bl_gemv_batch_static(const bl_gemv_item* items, int32_t count, int64_t M, void* stream) {
    bl::DecodeBatch b;
    const bl_status st = fill_gemv_batch(items, count, M, b);
    if (st != BL_OK) return st;
    drop_stale_hip_error();
    unsigned long long* ws = nullptr;
    const hipError_t e = scratch_for_current_device(static_cast<hipStream_t>(stream), &ws);
    if (e != hipSuccess) return hip_status(e);
    b.ws = ws;
    // the balanced form would use 64 words per workgroup: more workgroups than the array holds is an error here,
    // not a silent change of kernel
    if (M == 1 && bl::decode_split_grid(b, false) > BL_STATIC_WS_WGS) return BL_ERR_WORKSPACE;
    return hip_status(bl::launch_decode(b, (int)M, false, static_cast<hipStream_t>(stream)));
}

bl_status bl_decode_batch(const bl_decode_item* items, int32_t count, int64_t M, void* workspace_dev, void* stream) {
    if (!items) return BL_ERR_NULL;
    if (count < 1 || count > BL_MAX_BATCH) return BL_ERR_COUNT;
    if (M < 1 || M > BL_MAX_GEMV_M) return BL_ERR_M_RANGE;
    if (workspace_dev && !aligned(workspace_dev, 256)) return BL_ERR_ALIGN;
    bl::DecodeBatch b;
    memset(&b, 0, sizeof b);
    b.ws = static_cast<unsigned long long*>(workspace_dev);
    int64_t max_Kp = 0;
    for (int i = 0; i < count; ++i) {
        const bl_decode_item& it = items[i];
        if (!it.x_dev || !it.packed_dev || !it.desc || !it.out_dev) return BL_ERR_NULL;
        if (it.dt != BL_F32 && it.dt != BL_BF16) return BL_ERR_DTYPE;
        if (it.dt != items[0].dt) return BL_ERR_DTYPE;   // one activation dtype per launch
        bl_status s = check_desc(it.desc);
        if (s != BL_OK) return s;
        if (it.ldx < it.desc->K) return BL_ERR_SHAPE;
        if (!aligned(it.x_dev, it.dt == BL_F32 ? 4 : 2) || !aligned(it.packed_dev, 16) || !aligned(it.out_dev, 4) ||
            (it.acc_dev && !aligned(it.acc_dev, 4)) || (it.q_dev && !aligned(it.q_dev, 16)) ||
            (it.a_scale_dev && !aligned(it.a_scale_dev, 4)) || (it.q_sum_dev && !aligned(it.q_sum_dev, 4)))
            return BL_ERR_ALIGN;
        bl::DecodeProblem& p = b.p[i];
        p = make_decode_problem(it.packed_dev, it.desc, it.out_dev, it.acc_dev);
        p.x = it.x_dev;
        p.ldx = it.ldx;
        p.q_out = it.q_dev;
        p.a_scale_out = it.a_scale_dev;
        p.q_sum_out = it.q_sum_dev;
        const bool vec = (it.desc->K % 8 == 0) && (it.ldx % 8 == 0) && aligned(it.x_dev, 16);
        p.x_flags = (it.dt == BL_BF16 ? 1 : 0) | (vec ? 2 : 0);
        if (it.desc->Kp > max_Kp) max_Kp = it.desc->Kp;
    }
    if (bl::decode_lds_bytes((int)M, max_Kp, true) > (size_t)bl::kMaxDecodeLds) return BL_ERR_SHAPE;
    b.count = count;
    drop_stale_hip_error();
    return hip_status(bl::launch_decode(b, (int)M, true, static_cast<hipStream_t>(stream)));
}

bl_status bl_gemm(const void* packed_dev, const bl_packed_desc* d, const int8_t* q_dev, const float* a_scale_dev,
                  const int32_t* q_sum_dev, int64_t M, float* out_dev, int32_t* acc_dev, void* stream) {
    bl_status s = check_product_args(packed_dev, d, q_dev, a_scale_dev, q_sum_dev, M, out_dev, acc_dev);
    if (s != BL_OK) return s;
    if (M > BL_MAX_GEMM_M) return BL_ERR_SHAPE;
    bl::GemmProblem p = make_problem(packed_dev, d, q_dev, a_scale_dev, q_sum_dev, out_dev, acc_dev);
    drop_stale_hip_error();
    return hip_status(bl::launch_gemm(p, M, static_cast<hipStream_t>(stream)));
}

bl_status bl_gemm_batch(const bl_gemv_item* items, int32_t count, int64_t M, void* stream) {
    if (!items) return BL_ERR_NULL;
    if (count < 1 || count > BL_MAX_GEMM_BATCH) return BL_ERR_COUNT;
    if (M < 1 || M > BL_MAX_GEMM_M) return BL_ERR_SHAPE;
    bl::GemmProblem ps[BL_MAX_GEMM_BATCH];
    for (int i = 0; i < count; ++i) {
        const bl_gemv_item& it = items[i];
        bl_status s = check_product_args(it.packed_dev, it.desc, it.q_dev, it.a_scale_dev, it.q_sum_dev, M, it.out_dev,
                                         it.acc_dev);
        if (s != BL_OK) return s;
        ps[i] = make_problem(it.packed_dev, it.desc, it.q_dev, it.a_scale_dev, it.q_sum_dev, it.out_dev, it.acc_dev);
    }
    drop_stale_hip_error();
    return hip_status(bl::launch_gemm_batch(ps, count, M, static_cast<hipStream_t>(stream)));
}

bl_status bl_norm_quant(const bl_norm_quant_args* a, void* stream) {
    if (!a || (!a->gamma_dev && a->mode != BL_NORM_PREMULTIPLIED)) return BL_ERR_NULL;
    const bool quantize = a->q_dev != nullptr;
    if (quantize != (a->a_scale_dev != nullptr) || (!quantize && a->q_sum_dev)) return BL_ERR_NULL;
    switch (a->mode) {
        case BL_NORM_PLAIN: if (!a->a_dev) return BL_ERR_NULL; break;
        case BL_NORM_RESIDUAL: if (!a->h_dev) return BL_ERR_NULL; break;
        case BL_NORM_GATED: if (!a->a_dev || !a->b_dev) return BL_ERR_NULL; break;
        case BL_NORM_PREMULTIPLIED:
            if (!a->a_dev || !a->scratch_dev) return BL_ERR_NULL;
            if (a->pieces < 1 || a->M != 1 || a->K > BL_MAX_K) return BL_ERR_SHAPE;
            break;
        default: return BL_ERR_SHAPE;
    }
    if (a->M < 1 || a->K < 1 || (a->K > BL_NORM_MAX_K && a->mode != BL_NORM_PREMULTIPLIED)) return BL_ERR_SHAPE;
    if (quantize && (a->Kp < a->K || a->Kp % 4 != 0 || a->Kp > BL_MAX_K)) return BL_ERR_SHAPE;
    if (!aligned(a->a_dev, 4) || !aligned(a->b_dev, 4) || !aligned(a->h_dev, 4) || !aligned(a->gamma_dev, 4) ||
        !aligned(a->q_dev, 4) || !aligned(a->a_scale_dev, 4) || !aligned(a->q_sum_dev, 4) || !aligned(a->y_dev, 4) ||
        !aligned(a->scratch_dev, 8))
        return BL_ERR_ALIGN;
    drop_stale_hip_error();
    return hip_status(bl::launch_norm_quant(*a, static_cast<hipStream_t>(stream)));
}

bl_status bl_decode_norm_batch(const bl_decode_norm_item* items, int32_t count, void* workspace_dev, void* stream) {
    if (!items) return BL_ERR_NULL;
    if (count < 1 || count > BL_MAX_BATCH) return BL_ERR_COUNT;
    if (workspace_dev && !aligned(workspace_dev, 256)) return BL_ERR_ALIGN;
    bl::DecodeBatch b;
    memset(&b, 0, sizeof b);
    b.ws = static_cast<unsigned long long*>(workspace_dev);
    int64_t max_Kp = 0;
    for (int i = 0; i < count; ++i) {
        const bl_decode_norm_item& it = items[i];
        if (!it.x_dev || !it.packed_dev || !it.desc || !it.out_dev) return BL_ERR_NULL;
        if (!it.gamma_dev && !it.ss_in_dev) return BL_ERR_NULL;            // one of the two forms of the norm
        if (it.glu_gamma_dev && !it.ss_out_dev) return BL_ERR_NULL;
        bl_status s = check_desc(it.desc);
        if (s != BL_OK) return s;
        if (it.desc->K % 8 != 0 || it.desc->K > BL_DECODE_NORM_MAX_K) return BL_ERR_SHAPE;
        if (it.h_out_dev && (it.h_out_dev == it.x_dev || it.h_out_dev == it.delta_dev)) return BL_ERR_SHAPE;
        if (!it.gamma_dev && (it.delta_dev || it.h_out_dev || it.ss_count < 1)) return BL_ERR_SHAPE;
        if (it.gamma_dev && it.ss_in_dev) return BL_ERR_SHAPE;
        if ((it.gamma_dev != nullptr) != (items[0].gamma_dev != nullptr) ||
            (it.glu_gamma_dev != nullptr) != (items[0].glu_gamma_dev != nullptr))
            return BL_ERR_SHAPE;                                           // one form per launch
        if (it.glu_gamma_dev && it.desc->N % BL_TILE_N != 0) return BL_ERR_SHAPE;
        if (!aligned(it.x_dev, 16) || !aligned(it.gamma_dev, 16) || !aligned(it.delta_dev, 16) || !aligned(it.h_out_dev, 16) ||
            !aligned(it.packed_dev, 16) || !aligned(it.out_dev, 4) || !aligned(it.acc_dev, 4) || !aligned(it.q_dev, 16) ||
            !aligned(it.a_scale_dev, 4) || !aligned(it.q_sum_dev, 4) || !aligned(it.ss_in_dev, 8) ||
            !aligned(it.glu_gamma_dev, 4) || !aligned(it.ss_out_dev, 8))
            return BL_ERR_ALIGN;
        bl::DecodeProblem& p = b.p[i];
        p = make_decode_problem(it.packed_dev, it.desc, it.out_dev, it.acc_dev);
        p.x = it.x_dev;
        p.ldx = it.desc->K;
        p.q_out = it.q_dev;
        p.a_scale_out = it.a_scale_dev;
        p.q_sum_out = it.q_sum_dev;
        p.x_flags = 2;   // fp32, vector loads: the row lives in registers
        p.gamma = it.gamma_dev;
        p.delta = it.delta_dev;
        p.h_out = it.h_out_dev;
        p.eps = it.eps;
        p.ss_in = reinterpret_cast<const float2*>(it.ss_in_dev);
        p.ss_count = it.ss_count;
        p.glu_gamma = it.glu_gamma_dev;
        p.ss_out = reinterpret_cast<float2*>(it.ss_out_dev);
        p.w_scale2 = it.w_scale_up;
        if (it.desc->Kp > max_Kp) max_Kp = it.desc->Kp;
    }
    if (bl::decode_lds_bytes(1, max_Kp, true) > (size_t)bl::kMaxDecodeLds) return BL_ERR_SHAPE;
    b.count = count;
    drop_stale_hip_error();
    return hip_status(bl::launch_decode(b, 1, true, static_cast<hipStream_t>(stream)));
}

bl_status bl_rope_table(float* table_dev, int32_t head_dim, int32_t max_pos, double theta, void* stream) {
    if (!table_dev) return BL_ERR_NULL;
    if (head_dim < 2 || head_dim > BL_ATTN_MAX_HEAD_DIM || head_dim % 2 != 0 || max_pos < 1 || !(theta > 0.0))
        return BL_ERR_SHAPE;
    if (!aligned(table_dev, 8)) return BL_ERR_ALIGN;
    drop_stale_hip_error();
    return hip_status(bl::launch_rope_table(table_dev, head_dim, max_pos, theta, static_cast<hipStream_t>(stream)));
}

static bool attn_shape_ok(int32_t n_heads, int32_t head_dim, int32_t max_pos) {
    return n_heads >= 1 && n_heads <= 65535 && head_dim >= 4 && head_dim <= BL_ATTN_MAX_HEAD_DIM && head_dim % 4 == 0 &&
           max_pos >= 1 && bl::attn_chunks(max_pos) <= 65535;
}

uint64_t bl_attn_scratch_bytes(int32_t n_heads, int32_t head_dim, int32_t max_pos) {
    if (!attn_shape_ok(n_heads, head_dim, max_pos)) return 0;
    // per (head, chunk): head_dim weighted values, the chunk's maximum and sum; then one ticket counter per head
    return (uint64_t)n_heads * (uint64_t)bl::attn_chunks(max_pos) * (uint64_t)(head_dim + 2) * sizeof(float) +
           (uint64_t)n_heads * sizeof(uint32_t);
}

bl_status bl_attn_decode(const bl_attn_args* a, void* stream) {
    if (!a || !a->q_lin_dev || !a->k_lin_dev || !a->v_lin_dev || !a->pos_dev || !a->rope_table_dev || !a->k_cache_dev ||
        !a->v_cache_dev || !a->out_dev || !a->scratch_dev)
        return BL_ERR_NULL;
    if (!attn_shape_ok(a->n_heads, a->head_dim, a->max_pos)) return BL_ERR_SHAPE;
    if (!aligned(a->q_lin_dev, 4) || !aligned(a->k_lin_dev, 4) || !aligned(a->v_lin_dev, 4) || !aligned(a->pos_dev, 4) ||
        !aligned(a->rope_table_dev, 8) || !aligned(a->k_cache_dev, 16) || !aligned(a->v_cache_dev, 16) ||
        !aligned(a->out_dev, 4) || !aligned(a->scratch_dev, 16))
        return BL_ERR_ALIGN;
    drop_stale_hip_error();
    return hip_status(bl::launch_attn_decode(*a, static_cast<hipStream_t>(stream)));
}

static bool prefill_shape_ok(int32_t n_heads, int32_t head_dim, int32_t pos0, int32_t M) {
    return pos0 >= 0 && M >= 1 && M <= 65535 && (int64_t)pos0 + M <= INT32_MAX / 2 && attn_shape_ok(n_heads, head_dim, pos0 + M);
}

uint64_t bl_attn_prefill_scratch_bytes(int32_t n_heads, int32_t head_dim, int32_t pos0, int32_t M) {
    if (!prefill_shape_ok(n_heads, head_dim, pos0, M)) return 0;
    if (head_dim <= BL_ATTN_BLOCK_MAX_HEAD_DIM) return 16;   // the matrix-core kernel keeps everything in registers and LDS
    const uint64_t per_query = (uint64_t)n_heads * (uint64_t)bl::attn_chunks(pos0 + M) * (uint64_t)(head_dim + 2) + (uint64_t)n_heads;
    return per_query * (uint64_t)M * sizeof(float);
}

bl_status bl_attn_prefill(const bl_attn_prefill_args* a, void* stream) {
    if (!a || !a->q_lin_dev || !a->k_lin_dev || !a->v_lin_dev || !a->rope_table_dev || !a->k_cache_dev || !a->v_cache_dev ||
        !a->out_dev || !a->scratch_dev)
        return BL_ERR_NULL;
    if (!prefill_shape_ok(a->n_heads, a->head_dim, a->pos0, a->M) || !attn_shape_ok(a->n_heads, a->head_dim, a->max_pos) ||
        a->pos0 + a->M > a->max_pos)
        return BL_ERR_SHAPE;
    if (!aligned(a->q_lin_dev, 4) || !aligned(a->k_lin_dev, 8) || !aligned(a->v_lin_dev, 8) || !aligned(a->rope_table_dev, 8) ||
        !aligned(a->k_cache_dev, 16) || !aligned(a->v_cache_dev, 16) || !aligned(a->out_dev, 4) || !aligned(a->scratch_dev, 16))
        return BL_ERR_ALIGN;
    drop_stale_hip_error();
    return hip_status(bl::launch_attn_prefill(*a, static_cast<hipStream_t>(stream)));
}

bl_status bl_pos_advance(int32_t* pos_dev, void* stream) {
    if (!pos_dev) return BL_ERR_NULL;
    if (!aligned(pos_dev, 4)) return BL_ERR_ALIGN;
    drop_stale_hip_error();
    return hip_status(bl::launch_pos_advance(pos_dev, static_cast<hipStream_t>(stream)));
}

const char* bl_status_str(bl_status s) {
    switch (s) {
        case BL_OK: return "ok";
        case BL_ERR_NULL: return "a required pointer is NULL";
        case BL_ERR_SHAPE: return "shape or stride out of range";
        case BL_ERR_M_RANGE: return "M outside 1..8 for the decode product";
        case BL_ERR_BUF_SMALL: return "descriptor byte count does not match its shape";
        case BL_ERR_ALIGN: return "pointer not aligned as documented";
        case BL_ERR_DTYPE: return "unknown activation dtype";
        case BL_ERR_LAYOUT: return "unknown packed layout version";
        case BL_ERR_HIP: return "HIP launch failed";
        case BL_ERR_COUNT: return "batch count outside 1..8";
        case BL_ERR_WORKSPACE: return "the launch needs more scratch than the library's static array holds";
    }
    return "unknown status";
}

bl_status bl_set_tuning(const char* key, int32_t value) {
    if (!key) return BL_ERR_NULL;
    if (strcmp(key, "gemv_waves") == 0) {
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8 && value != 16) return BL_ERR_SHAPE;
        bl::set_gemv_waves(value);
        return BL_OK;
    }
    if (strcmp(key, "decode_stage") == 0) {
        if (value < 0 || value > 1) return BL_ERR_SHAPE;
        bl::set_decode_stage(value);
        return BL_OK;
    }
    if (strcmp(key, "gemm_mb") == 0) {
        if (value != 0 && !bl::gemm_form_exists(value)) return BL_ERR_SHAPE;
        bl::set_gemm_mb(value);
        return BL_OK;
    }
    if (strcmp(key, "attn_groups") == 0) {
        if (value < 0 || value > 65535) return BL_ERR_SHAPE;
        bl::set_attn_groups(value);
        return BL_OK;
    }
    if (strcmp(key, "decode_split") == 0) {
        if (value < -1 || value > 8) return BL_ERR_SHAPE;
        bl::set_decode_split(value);
        return BL_OK;
    }
    if (strcmp(key, "decode_publish") == 0) {
        if (value < -1 || value > 0) return BL_ERR_SHAPE;
        bl::set_decode_publish(value);
        return BL_OK;
    }
    if (strcmp(key, "decode_wait_limit") == 0) {
        if (value < 0) return BL_ERR_SHAPE;
        bl::set_decode_wait_limit(value);
        return BL_OK;
    }
    if (strcmp(key, "decode_stream") == 0) {
        if (value < -1 || value > 1) return BL_ERR_SHAPE;
        bl::set_decode_stream(value);
        return BL_OK;
    }
    if (strcmp(key, "decode_path") == 0) {
        if (value < 0 || value > 2) return BL_ERR_SHAPE;
        bl::set_decode_path(value);
        return BL_OK;
    }
    return BL_ERR_SHAPE;
}

int64_t bl_get_stat(const char* key) {
    if (key && strcmp(key, "split_launches") == 0) return bl::split_launches();
    return -1;
}

const char* bl_last_hip_error(void) { return hipGetErrorString(t_last_hip_error); }

const char* bl_last_kernel(void) {
    const bl::KernelNote& n = bl::t_kernel_note;
    if (!n.fmt) return "";
    // the note's format: %d = next value as a number, %b = next value as true / false (as profilers print the name)
    char* out = t_kernel_text;
    char* const end = t_kernel_text + sizeof t_kernel_text - 24;
    int next = 0;
    for (const char* f = n.fmt; *f && out < end; ++f) {
        if (f[0] == '%' && (f[1] == 'd' || f[1] == 'b') && next < 8) {
            const int v = n.v[next++];
            out += f[1] == 'd' ? snprintf(out, 16, "%d", v) : snprintf(out, 16, "%s", v ? "true" : "false");
            ++f;
        } else {
            *out++ = *f;
        }
    }
    snprintf(out, 24, " grid=%d", n.grid);
    return t_kernel_text;
}

const char* bl_version(void) { return "bitlinear-gfx950 0.2 (layouts 1, 2)"; }

}  // extern "C"
