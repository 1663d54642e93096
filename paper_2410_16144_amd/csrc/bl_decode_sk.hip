// Work-balanced decode product for one token: every workgroup streams the same number of weight
// tiles, whatever the shapes of the matrices in the launch (Section 2 of arXiv 2410.16144, I2_S
// form: codes back to weights in registers, multiply-add against int8 activations).
//
// The launch has a fixed number of workgroups (a multiple of the compute-unit count).  Each matrix
// gets a share of them in proportion to its tile count; inside a matrix, the tiles, in memory
// order (row block major, then K), are cut into equal contiguous chunks, one per workgroup, and
// the chunk is cut again into 16 contiguous pieces, one per wave.  A piece may begin and end in
// the middle of a row block:
//   * inside the workgroup the pieces of one row block meet in LDS (integer adds);
//   * a row block cut by a chunk boundary is finished through the caller's workspace: per row one
//     64-bit word, the tile count in its high bits and the signed partial sum in its low 40 bits,
//     so ONE returning atomic add per row both deposits a partial sum and tells the depositor
//     whether it was the last one; the last one writes the output and stores zero back.
// Integer addition is exact and order-free, so the result is bit-identical to the unsplit kernel.
#include "bl_decode_device.hpp"

namespace bl {

namespace {

constexpr int kSkMaxRb = 32;   // row blocks one chunk may touch (LDS: 256 bytes each)
constexpr int kSumBits = 40;   // low bits of a workspace word that hold the partial sum

// LAYOUT 2: TL2-coded tiles (plain form only).  NORM (fp32 rows only): 1 = RMSNorm folded into the fused quantizer,
// 2 = the row is already multiplied by its norm weight and sum(x^2) arrives in pieces.
// STREAM: weight tiles by streaming (nontemporal) loads, see load_weight_tile.
// GLU (with NORM 1): gated epilogue (see DecodeProblem).  It pairs lanes l and l + 32 of a row block, so ONE wave must
// finish all 64 rows of a shared row block: see the epilogue.
template <int U, bool FUSED, bool XBF16, int LAYOUT, int NORM, bool STREAM, bool GLU = false>
__global__ __launch_bounds__(kThreads, 8) void decode_sk_kernel(BL_FIRST_WG_PARAMS, const DecodeBatch b) {
    static_assert(LAYOUT == 1 || (LAYOUT == 2 && !FUSED), "the TL2 layout has the plain form only");
    static_assert(!GLU || NORM == 1, "the gated epilogue comes with the folded norm");
    static_assert(NORM == 0 || (FUSED && !XBF16 && LAYOUT == 1), "the norm is folded into the fused quantizer of fp32 rows");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ int tl2_lut[LAYOUT == 2 ? 32 : 1];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int blk = blockIdx.x;
    const DecodeProblem& p = b.p[BL_PROBLEM_OF(blk)];

    const int KC = p.KC, Kp = KC * kTileK;
    const int T = p.row_blocks * KC;                           // tiles of this matrix
    const int a = min((blk - p.first_wg) * p.chunk, T);        // this workgroup's tiles [a, e)
    const int e = min(a + p.chunk, T);
    if (a >= e) return;                                        // uniform: a workgroup without work
    const int per_wave = (e - a + kWaves - 1) / kWaves;
    const int t_wave = min(a + wave * per_wave, e);            // this wave's tiles [t_wave, t_wave + mine)
    const int mine = min(per_wave, e - t_wave);
    const int t_last = mine > 0 ? t_wave + mine - 1 : a;
    const int rb0 = a / KC, rb1 = (e - 1) / KC;                // row blocks the chunk touches

    int8_t* lds_q = reinterpret_cast<int8_t*>(smem);
    int* red = reinterpret_cast<int*>(smem + (FUSED ? Kp : 0));    // [row block - rb0][64]
    float* s_f = reinterpret_cast<float*>(red + kSkMaxRb * kWave);  // [16] maxima, then the scale
    int* s_i = reinterpret_cast<int*>(s_f + kWaves + 1);            // [16] partial sum(q)
    float* s_ss = reinterpret_cast<float*>(s_i + kWaves);           // [16] partial sums of squares (norm form)

    for (int i = tid; i < (rb1 - rb0 + 1) * kWave; i += kThreads) red[i] = 0;

    const uint4* __restrict__ wp = p.packed + lane;
    uint4 w[U];
    auto load_part = [&](int i0, int first, int last) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (u >= first && u < last) {
                // beyond the wave's piece: its own last tile again (a cache hit, no extra traffic); a wave without
                // tiles loads the chunk's first tile
                w[u] = load_weight_tile<STREAM>(wp + (int64_t)min(t_wave + i0 + u, t_last) * kWave);
            }
        }
    };
    auto load_batch = [&](int i0) { load_part(i0, 0, U); };
    // tiles that go in flight ahead of the quantizer (register budget; the norm form also holds gamma and delta)
    constexpr int kEarly = NORM == 1 ? U / 4 : U > 4 ? U / 2 : U;

    int qsum = 0;
    float scale = 0.0f;
    if constexpr (!FUSED) {
        load_batch(0);
        if constexpr (LAYOUT == 2) tl2_fill_table(tl2_lut, tid);   // signed weights: no sum(q) correction
        else qsum = p.q_sum[0];
        scale = p.a_scale[0];
        __syncthreads();   // red is zero before the first deposit (and the TL2 table is in place)
    } else {
        const bool vec = p.x_flags & 2;
        int holding_waves = kWaves;   // waves with a part of sum(q)
        if (vec && p.K <= 2 * kThreads * 8) {
            // The token row lives in the registers of the workgroup's leading waves (two vectors per thread).  Those
            // waves ask for it first (loads retire in order, so their wait for it leaves the tiles that follow in
            // flight).  The other waves have no part in the quantizer: they take its first barrier before they
            // queue up their own tile loads, so that it is not held up by requests that wait for room in the
            // compute unit's load queue, and then request all their tiles at once.  Two barriers on either path.
            holding_waves = row_threads(p.K) / kWave;
            if (wave < holding_waves) {
                const int holders = holding_waves * kWave;
                const int k0 = tid * 8, k1 = k0 + holders * 8;
                const bool h0 = k0 < p.K, h1 = k1 < p.K;
                Raw8<XBF16> r0 = load_raw8<XBF16>(p.x, h0 ? k0 : 0), r1 = load_raw8<XBF16>(p.x, h1 ? k1 : 0);
                if constexpr (NORM == 2) {
                    load_part(0, 0, kEarly);
                    const float ss = wave_sum_f(norm_pieces(p.ss_in, p.ss_count, tid, holders));
                    if (lane == 0) s_ss[wave] = ss;
                } else if constexpr (NORM == 1) {
                    {
                        const Raw8<false> g0 = load_raw8<false>(p.gamma, h0 ? k0 : 0), g1 = load_raw8<false>(p.gamma, h1 ? k1 : 0);
                        Raw8<false> d0 = g0, d1 = g1;
                        if (p.delta) {
                            d0 = load_raw8<false>(p.delta, h0 ? k0 : 0);
                            d1 = load_raw8<false>(p.delta, h1 ? k1 : 0);
                        }
                        load_part(0, 0, kEarly);
                        float ss = norm_fold(r0, r1, g0, g1, d0, d1, h0, h1, k0, k1, p.delta != nullptr,
                                             blk == p.first_wg ? p.h_out : nullptr);
                        ss = wave_sum_f(ss);
                        if (lane == 0) s_ss[wave] = ss;
                    }
                } else {
                    load_part(0, 0, kEarly);
                }
                row_absmax_to_lds<XBF16>(r0, r1, h0, h1, s_f, lane, wave);
                __syncthreads();
                row_quantize_to_lds<XBF16>(r0, r1, h0, h1, k0, k1, holders, p.K, Kp, lds_q, s_f, s_i, tid, lane, wave);
                __syncthreads();
                load_part(0, kEarly, U);
            } else {
                __syncthreads();
                load_batch(0);
                __syncthreads();
            }
        } else {
            if (vec) quantize_rows_to_lds<1, XBF16, true, true>(p, lds_q, s_f, s_i, tid, lane, wave);
            else quantize_rows_to_lds<1, XBF16, false>(p, lds_q, s_f, s_i, tid, lane, wave);
            load_batch(0);
        }
        for (int w16 = 0; w16 < holding_waves; ++w16) qsum += s_i[w16];
        scale = s_f[kWaves];
        if constexpr (NORM != 0) scale *= norm_scalar(s_ss, holding_waves, p.K, p.eps);
        if (blk == p.first_wg) {   // optional copy-out of the quantizer's results
            if (p.q_out) {
                for (int i = tid; i < Kp / 4; i += kThreads)
                    reinterpret_cast<int32_t*>(p.q_out)[i] = reinterpret_cast<const int32_t*>(lds_q)[i];
            }
            if (tid == 0) {
                if (p.a_scale_out) p.a_scale_out[0] = scale;
                if (p.q_sum_out) p.q_sum_out[0] = qsum;
            }
        }
    }

    Acc<1> acc;
    acc.lo[0] = acc.hi[0] = 0;
    int rb = min(t_wave, T - 1) / KC;
    int kc = t_wave - rb * KC;
    auto deposit = [&]() {
        __hip_atomic_fetch_add(&red[(rb - rb0) * kWave + lane], acc.lo[0] + (acc.hi[0] >> 2), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_WORKGROUP);   // hi: exact multiple of 4
        acc.lo[0] = acc.hi[0] = 0;
    };
    if (mine > 0) {
        for (int i0 = 0;;) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (i0 + u < mine) {
                    if (kc == KC) {   // the piece runs on into the next row block
                        deposit();
                        ++rb;
                        kc = 0;
                    }
                    if constexpr (LAYOUT == 2) tl2_tile_mac(w[u], p.q + kc * kTl2QWords, tl2_lut, acc.lo[0]);
                    else if constexpr (FUSED) tile_mac<1>(w[u], reinterpret_cast<const int32_t*>(lds_q) + kc * 16, Kp / 4, acc);
                    else tile_mac<1>(w[u], p.q + kc * 16, Kp / 4, acc);
                    ++kc;
                }
                if constexpr (LAYOUT == 1) __builtin_amdgcn_sched_barrier(0);
            }
            i0 += U;
            if (i0 >= mine) break;
            load_batch(i0);
        }
        deposit();
    }
    __syncthreads();

    for (int r = rb0 + wave; r <= rb1; r += kWaves) {
        const int v = red[(r - rb0) * kWave + lane];
        const int t_first = r * KC, t_end = t_first + KC;
        int total = v;
        bool last = true;
        if (t_first < a || t_end > e) {   // uniform: the row block is shared with other workgroups
            const int cnt = min(e, t_end) - max(a, t_first);
            const int owner = p.first_wg + t_first / p.chunk;   // the workgroup that holds the block's first tile
            unsigned long long* slot = b.ws + (int64_t)owner * kWave + lane;
            const unsigned long long add = ((unsigned long long)cnt << kSumBits) + (unsigned long long)(long long)v;
            unsigned long long now =
                __hip_atomic_fetch_add(slot, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + add;
            if constexpr (GLU) {
                // Per-row counts cannot serve here: the 64 words lie in four cache lines, so two depositors may each be
                // last on some of them, and the gated epilogue needs ONE wave with all 64 rows.  So: deposit (a
                // returning operation: it has been performed where every die sees it once its value is back), wait
                // for all 64 to return, THEN draw a ticket of `cnt` tiles from one word per row block.  Whoever's
                // ticket completes the block's KC tiles reads the 64 sums -- every depositor's were performed before
                // its ticket -- and puts words and ticket back to zero.  Nobody waits for anybody.
                asm volatile("s_waitcnt vmcnt(0)" ::"v"(now) : "memory");
                unsigned int* ticket = reinterpret_cast<unsigned int*>(reinterpret_cast<char*>(b.ws) + BL_WORKSPACE_BYTES - kPubBytes) + owner;
                unsigned int drawn = 0;
                if (lane == 0) drawn = __hip_atomic_fetch_add(ticket, (unsigned)cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + (unsigned)cnt;
                last = __builtin_amdgcn_readfirstlane(drawn) == (unsigned)KC;   // uniform
                if (last) {
                    now = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (lane == 0) __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                total = (int)((long long)(now << (64 - kSumBits)) >> (64 - kSumBits));
            } else {
                const long long sum = (long long)(now << (64 - kSumBits)) >> (64 - kSumBits);
                last = (long long)((now - (unsigned long long)sum) >> kSumBits) == KC;
                total = (int)sum;
                if (last) __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        const int row = r * kTileN + lane;
        if constexpr (GLU) {
            if (last) {   // uniform: the whole wave holds the block's 64 complete sums
                total -= qsum;
                // lanes 0-31: gate rows, lanes 32-63: the up rows of the same 32 outputs
                const float val = (float)total * ((lane < 32 ? p.w_scale : p.w_scale2) * scale);
                const float up = __shfl_xor(val, 32);
                const int n = r * 32 + (lane & 31);
                float x = 0.0f, z = 0.0f;
                if (lane < 32 && n < p.N / 2) {
                    x = silu(val) * up;
                    z = x * p.glu_gamma[n];
                    p.out[n] = z;
                }
                const float ss = wave_sum_f(x * x), zmax = wave_max(fabsf(z));
                if (lane == 0) p.ss_out[r] = make_float2(ss, zmax);
                if (p.acc && row < p.N) p.acc[row] = total;
            }
        } else if (last && row < p.N) {
            total -= qsum;
            p.out[row] = (float)total * (p.w_scale * scale);
            if (p.acc) p.acc[row] = total;
        }
    }
}

template <auto Kernel>
hipError_t launch_sk_kernel(const DecodeBatch& b, size_t lds, hipStream_t s) {
    static LdsCeiling ceiling;   // per kernel
    const hipError_t e = ceiling.ensure(reinterpret_cast<const void*>(Kernel));
    if (e != hipSuccess) return e;
    const FirstWgs first(b);
    Kernel<<<dim3((unsigned)b.total_wgs), dim3(kThreads), lds, s>>>(BL_FIRST_WG_ARGS(first), b);
    return hipGetLastError();
}

template <int U, bool FUSED, bool XBF16, int LAYOUT = 1, int NORM = 0, bool GLU = false>
hipError_t launch_sk(const DecodeBatch& b, size_t lds, hipStream_t s) {
    note_kernel("decode_sk_kernel<%d, %b, %b, %d, %d, %b, %b>", b.total_wgs, U, FUSED, XBF16, LAYOUT, NORM, b.stream != 0, GLU);
    return b.stream ? launch_sk_kernel<&decode_sk_kernel<U, FUSED, XBF16, LAYOUT, NORM, true, GLU>>(b, lds, s)
                    : launch_sk_kernel<&decode_sk_kernel<U, FUSED, XBF16, LAYOUT, NORM, false, GLU>>(b, lds, s);
}

int g_split = 0;   // -1 never, 0 automatic, n > 0: n workgroups per compute unit
int64_t g_split_launches = 0;

}  // namespace

// Compute units of the current device (cached per device); 0 if the runtime cannot tell.
int compute_unit_count() {
    constexpr int kMaxDevices = 64;
    static int cached[kMaxDevices];
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    if (cached[dev] > 0) return cached[dev];
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 0;
    cached[dev] = n;
    return n;
}

void set_decode_split(int v) { g_split = v; }
int64_t split_launches() { return g_split_launches; }

// The workgroups a balanced launch of this batch would have (each uses 64 workspace words), or 0 when the balanced
// form is not chosen by launch size (the caller then uses the row-block kernels).  Shapes only: no side effects.
int decode_split_grid(const DecodeBatch& b, bool fused) {
    if (g_split < 0 || !b.ws) return 0;
    const bool glu = b.p[0].glu_gamma != nullptr;
    // The gated launch takes the balanced form only when it is forced (bl_set_tuning "decode_split" > 0): measured on the
    // gate/up launches of the twelve Appendix-A shapes it is ahead on two (3.8B: 7.3 -> 6.1 us, 30B: 13.1 -> 12.4) and
    // behind on the rest (7B: 8.3 -> 10.2), where the row-block kernel with two row blocks per workgroup streams as fast.
    if (glu && (b.count != 1 || g_split == 0)) return 0;
    const int cus = compute_unit_count();
    if (cus <= 0) return 0;
    int64_t total = 0;
    for (int i = 0; i < b.count; ++i) {
        const int64_t t = (int64_t)b.p[i].row_blocks * b.p[i].KC;
        if (t > (1 << 30)) return 0;
        total += t;
    }
    // Measured on MI355X (decoder layers of 0.7B to 100B shapes): equal shares pay off between about 100 and 400
    // tiles per compute unit; below, the launch is latency-bound either way, above, many small workgroups
    // dispatched as others finish adapt better to compute units that stream at different speeds.
    const int64_t per_cu = total / cus;
    int mult = g_split;
    if (mult == 0 && b.layout == 2 && per_cu >= 32) {
        // TL2-coded tiles: the table lookups want as many waves per compute unit as fit, and with two workgroups per
        // unit the balanced form stays the faster one on the largest layers too (100B-shape layer: 81 against 85 us)
        mult = 2;
    } else if (mult == 0) {
        if (per_cu > 400) return 0;
        if (per_cu < (fused ? 100 : 32)) {
            // small launches: worth it only where whole row blocks cannot even occupy every compute unit
            int64_t row_blocks = 0;
            for (int i = 0; i < b.count; ++i) row_blocks += b.p[i].row_blocks;
            if (row_blocks >= cus || per_cu < 8) return 0;
            mult = 1;
        } else {
            mult = (!fused && per_cu <= 250) ? 2 : 1;
        }
    }
    const int64_t grid = (int64_t)cus * mult;
    // (the gated form keeps one ticket word per workgroup in the workspace's tail, behind the sums)
    if (glu && grid * kWave * 8 > BL_WORKSPACE_BYTES - kPubBytes) return 0;
    if (grid > BL_MAX_SPLIT_WGS || b.count > grid) return 0;
    if (total < grid * 8) return 0;   // under 8 tiles per workgroup: nothing to balance
    return (int)grid;
}

// Plans the balanced launch.  Returns false when the balanced form does not apply (the caller then
// uses the row-block kernels): tiny launches, shapes whose chunks would touch too many row blocks.
bool plan_decode_split(DecodeBatch& b, bool fused, int& tiles_per_wave) {
    const int grid = decode_split_grid(b, fused);
    if (grid <= 0) return false;
    int64_t T[BL_MAX_BATCH], total = 0;
    for (int i = 0; i < b.count; ++i) {
        T[i] = (int64_t)b.p[i].row_blocks * b.p[i].KC;
        total += T[i];
    }
    int g[BL_MAX_BATCH], used = 0;
    for (int i = 0; i < b.count; ++i) {
        g[i] = (int)(T[i] * grid / total);
        if (g[i] < 1) g[i] = 1;
        used += g[i];
    }
    auto chunk = [&](int i) { return (T[i] + g[i] - 1) / g[i]; };
    while (used < grid) {   // hand the remaining workgroups to the matrices with the largest chunks
        int best = 0;
        for (int i = 1; i < b.count; ++i)
            if (chunk(i) > chunk(best)) best = i;
        ++g[best];
        ++used;
    }
    while (used > grid) {   // rounding up to one workgroup overshot: take from the smallest chunks
        int best = -1;
        for (int i = 0; i < b.count; ++i)
            if (g[i] > 1 && (best < 0 || chunk(i) < chunk(best))) best = i;
        if (best < 0) return false;
        --g[best];
        --used;
    }
    int first = 0;
    int64_t max_chunk = 0;
    for (int i = 0; i < b.count; ++i) {
        const int64_t c = chunk(i);
        if (c / b.p[i].KC + 2 > kSkMaxRb) return false;
        b.p[i].chunk = (int32_t)c;
        b.p[i].first_wg = first;
        first += g[i];
        if (c > max_chunk) max_chunk = c;
    }
    b.total_wgs = grid;
    ++g_split_launches;
    tiles_per_wave = (int)((max_chunk + kWaves - 1) / kWaves);
    return true;
}

hipError_t launch_decode_split(const DecodeBatch& b, int tiles_per_wave, bool fused, hipStream_t s) {
    int64_t max_Kp = 0;
    for (int i = 0; i < b.count; ++i) max_Kp = (int64_t)b.p[i].KC * kTileK > max_Kp ? (int64_t)b.p[i].KC * kTileK : max_Kp;
    const size_t lds = (size_t)(fused ? max_Kp : 0) + (size_t)kSkMaxRb * kWave * 4 + (size_t)(3 * kWaves + 1) * 4;
    if (lds > (size_t)kMaxDecodeLds) return hipErrorInvalidValue;
    const bool bf16 = b.p[0].x_flags & 1;
    const bool small = tiles_per_wave <= 4;
    if (b.layout == 2) return small ? launch_sk<4, false, true, 2>(b, lds, s) : launch_sk<8, false, true, 2>(b, lds, s);
    if (!fused) return small ? launch_sk<4, false, true>(b, lds, s) : launch_sk<8, false, true>(b, lds, s);
    if (bf16) return small ? launch_sk<4, true, true>(b, lds, s) : launch_sk<8, true, true>(b, lds, s);
    if (b.p[0].gamma && b.p[0].glu_gamma)
        return small ? launch_sk<4, true, false, 1, 1, true>(b, lds, s) : launch_sk<8, true, false, 1, 1, true>(b, lds, s);
    if (b.p[0].gamma) return small ? launch_sk<4, true, false, 1, 1>(b, lds, s) : launch_sk<8, true, false, 1, 1>(b, lds, s);
    if (b.p[0].ss_in) return small ? launch_sk<4, true, false, 1, 2>(b, lds, s) : launch_sk<8, true, false, 1, 2>(b, lds, s);
    return small ? launch_sk<4, true, false>(b, lds, s) : launch_sk<8, true, false>(b, lds, s);
}

}  // namespace bl
