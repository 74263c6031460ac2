// GPU tasks of the AoT multi-stream DAG executor: fp32 NCHW kernels for gfx950 (wave64).
//
// The Nimble paper (arXiv 2012.02732) ships no kernels of its own: it replays the base
// framework's operators unchanged (Section 5, "Experimental Setup"). These are the
// operators of its benchmark networks, written for CDNA4.
//
// Every operator is written once as a *tile function*: the share of one 256-thread
// workgroup, addressed by a linear tile index. Two kinds of kernels are built from them:
//   * one stand-alone kernel per tile function (grid = number of tiles), taking ONE
//     by-value argument struct so that the task table can hold a ready-made argument
//     block per task (Section 4.1: kernel arguments are prepared once, ahead of time);
//   * the device-resident replay kernel at the end of this file, in which persistent
//     workgroups walk the recorded task schedule themselves.
//
// Sizing rule that differs from usual throughput tuning: tasks are small (tens of
// thousands of elements) and are meant to run next to sibling tasks of other streams
// (Section 2, "GPU Streams"), so grids are sized by the work, never "fill the chip".
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <type_traits>

#include "ng_device.h"
#include "ng_internal.h"

namespace ng {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// LDS floats every workgroup owns: the largest user is the conv3x3 input patch (4 x 33 x 34).
constexpr int kSmemFloats = 4 * 33 * 34;

// ------------------------------------------------------------------------------------
// bn_act / relu: y = x * s[c] + t[c] (s, t folded from gamma, beta, mean, var), optional ReLU
// ------------------------------------------------------------------------------------
__device__ __forceinline__ void bn_coeff(const BnArgs& a, int c, float& s, float& t) {
    if (a.gamma) {
        s = a.gamma[c] / sqrtf(a.var[c] + a.eps);
        t = a.beta[c] - a.mean[c] * s;
    } else {
        s = 1.f;
        t = 0.f;
    }
}

template <bool VEC4>
__device__ __forceinline__ void bn_act_tile(const BnArgs& a, int tile, float*) {
    const int i = tile * kBlock + threadIdx.x;
    if (VEC4) {                                   // HW % 4 == 0: a float4 never straddles channels
        const int e = i * 4;
        if (e >= a.total) return;
        float s, t;
        bn_coeff(a, (e / a.HW) % a.C, s, t);
        float4 v = *reinterpret_cast<const float4*>(a.x + e);
        v.x = fmaf(v.x, s, t), v.y = fmaf(v.y, s, t), v.z = fmaf(v.z, s, t), v.w = fmaf(v.w, s, t);
        if (a.relu) v.x = fmaxf(v.x, 0.f), v.y = fmaxf(v.y, 0.f), v.z = fmaxf(v.z, 0.f), v.w = fmaxf(v.w, 0.f);
        *reinterpret_cast<float4*>(a.y + e) = v;
    } else {
        if (i >= a.total) return;
        float s, t;
        bn_coeff(a, (i / a.HW) % a.C, s, t);
        float v = fmaf(a.x[i], s, t);
        a.y[i] = a.relu ? fmaxf(v, 0.f) : v;
    }
}

// ------------------------------------------------------------------------------------
// add_n: elementwise sum of k tensors, accumulated in argument order
// ------------------------------------------------------------------------------------
template <bool VEC4>
__device__ __forceinline__ void add_n_tile(const AddArgs& a, int tile, float*) {
    const int i = tile * kBlock + threadIdx.x;
    if (VEC4) {
        const int e = i * 4;
        if (e >= a.total) return;
        float4 acc = *reinterpret_cast<const float4*>(a.x[0] + e);
#pragma unroll
        for (int j = 1; j < NG_MAX_PREDS; ++j) {
            if (j >= a.k) break;
            const float4 v = *reinterpret_cast<const float4*>(a.x[j] + e);
            acc.x += v.x, acc.y += v.y, acc.z += v.z, acc.w += v.w;
        }
        *reinterpret_cast<float4*>(a.y + e) = acc;
    } else {
        if (i >= a.total) return;
        float acc = a.x[0][i];
#pragma unroll
        for (int j = 1; j < NG_MAX_PREDS; ++j) {
            if (j >= a.k) break;
            acc += a.x[j][i];
        }
        a.y[i] = acc;
    }
}

// ------------------------------------------------------------------------------------
// concat: output channel block j = channels [lo_j, lo_j + cnt_j) of input j
// ------------------------------------------------------------------------------------
template <bool VEC4>
__device__ __forceinline__ void concat_tile(const ConcatArgs& a, int tile, float*) {
    const int i = tile * kBlock + threadIdx.x;
    const int e = VEC4 ? i * 4 : i;
    if (e >= a.total) return;
    const int plane = e / a.HW, pix = e - plane * a.HW;
    const int n = plane / a.C, c = plane - n * a.C;
    const float* base = a.x[0];
    int cin = a.cin[0], lo = a.lo[0], first = a.first[0];
#pragma unroll
    for (int q = 1; q < NG_MAX_PREDS; ++q)
        if (q < a.k && c >= a.first[q]) base = a.x[q], cin = a.cin[q], lo = a.lo[q], first = a.first[q];
    const float* src = base + ((size_t)(n * cin + lo + c - first)) * a.HW + pix;
    if (VEC4)
        *reinterpret_cast<float4*>(a.y + e) = *reinterpret_cast<const float4*>(src);
    else
        a.y[e] = *src;
}

// ------------------------------------------------------------------------------------
// pool3x3: max (out-of-bounds taps ignored) or average over the in-bounds taps
// ------------------------------------------------------------------------------------
__device__ __forceinline__ void pool3x3_tile(const PoolArgs& a, int tile, float*) {
    const int i = tile * kBlock + threadIdx.x;
    if (i >= a.total) return;
    const int ow = i % a.Wo, t = i / a.Wo;
    const int oh = t % a.Ho, plane = t / a.Ho;
    const float* src = a.x + (size_t)plane * a.H * a.W;
    const int r0 = oh * a.stride - a.pad, c0 = ow * a.stride - a.pad;
    float acc = a.mode == 0 ? -INFINITY : 0.f;
    int cnt = 0;
#pragma unroll
    for (int dr = 0; dr < 3; ++dr)
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) {
            const int r = r0 + dr, c = c0 + dc;
            if (r >= 0 && r < a.H && c >= 0 && c < a.W) {
                const float v = src[r * a.W + c];
                acc = a.mode == 0 ? fmaxf(acc, v) : acc + v;
                ++cnt;
            }
        }
    a.y[i] = a.mode == 0 ? acc : acc / (float)cnt;
}

// ------------------------------------------------------------------------------------
// dwconv: depthwise K x K, pad K/2, stride S
// ------------------------------------------------------------------------------------
template <int K, int S>
__device__ __forceinline__ void dwconv_tile(const DwArgs& a, int tile, float*) {
    const int i = tile * kBlock + threadIdx.x;
    if (i >= a.total) return;
    const int ow = i % a.Wo, t = i / a.Wo;
    const int oh = t % a.Ho, plane = t / a.Ho;
    const int c = plane % a.C;
    const float* src = a.x + (size_t)plane * a.H * a.W;
    const float* wt = a.w + c * K * K;
    const int r0 = oh * S - K / 2, c0 = ow * S - K / 2;
    float acc = 0.f;
#pragma unroll
    for (int dr = 0; dr < K; ++dr)
#pragma unroll
        for (int dc = 0; dc < K; ++dc) {
            const int r = r0 + dr, cc = c0 + dc;
            if (r >= 0 && r < a.H && cc >= 0 && cc < a.W) acc = fmaf(wt[dr * K + dc], src[r * a.W + cc], acc);
        }
    a.y[i] = acc;
}

// ------------------------------------------------------------------------------------
// global_avgpool: one wavefront per (n, c) plane, shuffle reduction across 64 lanes
// ------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

__device__ __forceinline__ void global_avgpool_tile(const GapArgs& a, int tile, float*) {
    const int lane = threadIdx.x & 63;
    const int plane = tile * (kBlock / 64) + (threadIdx.x >> 6);
    if (plane >= a.planes) return;
    const float* src = a.x + (size_t)plane * a.HW;
    float acc = 0.f;
    for (int p = lane; p < a.HW; p += 64) acc += src[p];
    acc = wave_sum(acc);
    if (lane == 0) a.y[plane] = acc / (float)a.HW;
}

// ------------------------------------------------------------------------------------
// fc (small batch): one wavefront per output feature; y[n][o] = <W[o], x[n]> + b[o]
// ------------------------------------------------------------------------------------
__device__ __forceinline__ void fc_gemv_tile(const FcArgs& a, int tile, float*) {
    const int lane = threadIdx.x & 63;
    const int o = tile * (kBlock / 64) + (threadIdx.x >> 6);
    if (o >= a.Cout) return;
    const float* wr = a.w + (size_t)o * a.Cin;
    for (int n = 0; n < a.N; ++n) {
        const float* xr = a.x + (size_t)n * a.Cin;
        float acc = 0.f;
        if ((a.Cin & 3) == 0) {
            for (int k = lane * 4; k < a.Cin; k += 256) {
                const float4 wv = *reinterpret_cast<const float4*>(wr + k);
                const float4 xv = *reinterpret_cast<const float4*>(xr + k);
                acc = fmaf(wv.x, xv.x, acc), acc = fmaf(wv.y, xv.y, acc);
                acc = fmaf(wv.z, xv.z, acc), acc = fmaf(wv.w, xv.w, acc);
            }
        } else {
            for (int k = lane; k < a.Cin; k += 64) acc = fmaf(wr[k], xr[k], acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) a.y[(size_t)n * a.Cout + o] = acc + a.b[o];
    }
}

// ------------------------------------------------------------------------------------
// conv1x1 (and large-batch fc) on the matrix cores: Y[Cout x cols] = W[Cout x Cin] * X[Cin x cols]
// with cols = N * HW. v_mfma_f32_16x16x4_f32: A fragment lane l -> A[l % 16][l / 16],
// B fragment lane l -> B[l / 16][l % 16], accumulator register r of lane l -> D[4 * (l / 16) + r][l % 16].
// A workgroup of four wavefronts (2 x 2) owns a TM x TN output tile; K is walked in
// slices of KC staged through LDS (A transposed to [k][m] so both fragments read rows).
// ------------------------------------------------------------------------------------
template <int TM, int TN, int KC>
__device__ __forceinline__ void conv1x1_mfma_tile(const PwArgs& a, int tile, float* smem) {
    constexpr int WM = TM / 2, WN = TN / 2;           // per-wavefront sub-tile
    constexpr int FM = WM / 16, FN = WN / 16;         // 16 x 16 fragments per wavefront
    constexpr int LDA = TM + 1, LDB = TN + 1;
    static_assert(KC * (LDA + LDB) <= kSmemFloats, "LDS budget");
    float* As = smem;                                 // [KC][LDA]
    float* Bs = smem + KC * LDA;                      // [KC][LDB]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int by = tile / a.tiles_n, bx = tile - by * a.tiles_n;
    const int m0 = by * TM, n0 = bx * TN;

    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int k0 = 0; k0 < a.Cin; k0 += KC) {
        // A slice: W[m0 + m][k0 + k] -> As[k][m]; consecutive threads walk k (contiguous in W)
        for (int e = tid; e < TM * KC; e += kBlock) {
            const int k = e % KC, m = e / KC;
            const int gm = m0 + m, gk = k0 + k;
            As[k * LDA + m] = (gm < a.Cout && gk < a.Cin) ? a.w[(size_t)gm * a.Cin + gk] : 0.f;
        }
        // B slice: X[k0 + k][n0 + n] -> Bs[k][n]; consecutive threads walk pixels
        for (int e = tid; e < TN * KC; e += kBlock) {
            const int n = e % TN, k = e / TN;
            const int col = n0 + n, gk = k0 + k;
            float v = 0.f;
            if (col < a.cols && gk < a.Cin) {
                const int img = col / a.HW, pix = col - img * a.HW;
                v = a.x[((size_t)img * a.Cin + gk) * a.HW + pix];
            }
            Bs[k * LDB + n] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < KC; kk += 4) {
            float af[FM], bf[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) af[i] = As[(kk + (lane >> 4)) * LDA + wm * WM + i * 16 + (lane & 15)];
#pragma unroll
            for (int j = 0; j < FN; ++j) bf[j] = Bs[(kk + (lane >> 4)) * LDB + wn * WN + j * 16 + (lane & 15)];
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int col = n0 + wn * WN + j * 16 + (lane & 15);
            if (col >= a.cols) continue;
            const int img = col / a.HW, pix = col - img * a.HW;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = m0 + wm * WM + i * 16 + 4 * (lane >> 4) + r;
                if (m < a.Cout) {
                    const float b = a.bias ? a.bias[m] : 0.f;
                    a.y[((size_t)img * a.Cout + m) * a.HW + pix] = acc[i][j][r] + b;
                }
            }
        }
}

// ------------------------------------------------------------------------------------
// conv3x3 dense on the vector ALUs: one thread = one output pixel x 8 output channels.
// Input patches go through LDS (4 input channels per slice); the weights a wavefront
// needs are the same for all of its lanes, so they are read through uniform addresses.
// TP = 16: the workgroup owns a 16 x 16 pixel tile and one group of 8 output channels.
// TP = 8 : each wavefront owns the same 8 x 8 pixel tile and its own group of 8 channels.
// Tile index = (image * co_groups + channel group) * tiles_xy + pixel tile.
// ------------------------------------------------------------------------------------
template <int TP, int S>
__device__ __forceinline__ void conv3x3_tile(const C3Args& a, int tile, float* smem) {
    constexpr int CIC = 4;                             // input channels per LDS slice
    constexpr int IW = (TP - 1) * S + 3;               // input patch edge
    constexpr int LDP = IW + 1;
    constexpr int GROUPS = TP == 16 ? 1 : 4;           // channel groups per workgroup
    constexpr int CO = 8;
    static_assert(CIC * IW * LDP <= kSmemFloats, "LDS budget");
    float* patch = smem;                               // [CIC][IW][LDP]

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int local = TP == 16 ? tid : (tid & 63);
    const int ty = local / TP, tx = local % TP;
    const int ptile = tile % a.tiles_xy, rest = tile / a.tiles_xy;
    const int cog = rest % a.co_groups, img = rest / a.co_groups;
    const int tile_y = ptile / a.tiles_x, tile_x = ptile - tile_y * a.tiles_x;
    const int oy = tile_y * TP + ty, ox = tile_x * TP + tx;
    const int co0 = (cog * GROUPS + (TP == 16 ? 0 : wave)) * CO;
    const int iy0 = tile_y * TP * S - a.pad, ix0 = tile_x * TP * S - a.pad;
    const float* xin = a.x + (size_t)img * a.Cin * a.H * a.W;

    float acc[CO];
#pragma unroll
    for (int j = 0; j < CO; ++j) acc[j] = 0.f;
    // clamped weight rows: out-of-range channels repeat the last one and are masked at the store
    const float* wrow[CO];
#pragma unroll
    for (int j = 0; j < CO; ++j) wrow[j] = a.w + (size_t)min(co0 + j, a.Cout - 1) * a.Cin * 9;

    for (int c0 = 0; c0 < a.Cin; c0 += CIC) {
        for (int e = tid; e < CIC * IW * IW; e += kBlock) {
            const int cx = e % IW, t = e / IW;
            const int cy = t % IW, ci = t / IW;
            const int gy = iy0 + cy, gx = ix0 + cx, gc = c0 + ci;
            float v = 0.f;
            if (gc < a.Cin && gy >= 0 && gy < a.H && gx >= 0 && gx < a.W) v = xin[((size_t)gc * a.H + gy) * a.W + gx];
            patch[(ci * IW + cy) * LDP + cx] = v;
        }
        __syncthreads();
        const int nci = min(CIC, a.Cin - c0);
        for (int ci = 0; ci < nci; ++ci) {
            float in[9];
#pragma unroll
            for (int dr = 0; dr < 3; ++dr)
#pragma unroll
                for (int dc = 0; dc < 3; ++dc) in[dr * 3 + dc] = patch[(ci * IW + ty * S + dr) * LDP + tx * S + dc];
#pragma unroll
            for (int j = 0; j < CO; ++j) {
                const float* wp = wrow[j] + (c0 + ci) * 9;
#pragma unroll
                for (int q = 0; q < 9; ++q) acc[j] = fmaf(wp[q], in[q], acc[j]);
            }
        }
        __syncthreads();
    }
    if (oy < a.Ho && ox < a.Wo) {
#pragma unroll
        for (int j = 0; j < CO; ++j)
            if (co0 + j < a.Cout) a.y[(((size_t)img * a.Cout + co0 + j) * a.Ho + oy) * a.Wo + ox] = acc[j];
    }
}

// ------------------------------------------------------------------------------------
// kernel table: id -> argument type, tile function, name
// ------------------------------------------------------------------------------------
template <int KID> struct KernelOf;
#define NG_KERNEL(KID, ARGS, CALL, NAME)                                                       \
    template <> struct KernelOf<KID> {                                                         \
        using Args = ARGS;                                                                     \
        static constexpr const char* name = NAME;                                              \
        static __device__ __forceinline__ void tile(const ARGS& a, int t, float* smem) { CALL(a, t, smem); } \
    };
NG_KERNEL(KID_BN, BnArgs, bn_act_tile<false>, "bn_act")
NG_KERNEL(KID_BN_V4, BnArgs, bn_act_tile<true>, "bn_act_v4")
NG_KERNEL(KID_ADD, AddArgs, add_n_tile<false>, "add_n")
NG_KERNEL(KID_ADD_V4, AddArgs, add_n_tile<true>, "add_n_v4")
NG_KERNEL(KID_CONCAT, ConcatArgs, concat_tile<false>, "concat")
NG_KERNEL(KID_CONCAT_V4, ConcatArgs, concat_tile<true>, "concat_v4")
NG_KERNEL(KID_POOL, PoolArgs, pool3x3_tile, "pool3x3")
#define NG_DW(K, S) dwconv_tile<K, S>
NG_KERNEL(KID_DW_K3S1, DwArgs, (NG_DW(3, 1)), "dwconv_k3s1")
NG_KERNEL(KID_DW_K3S2, DwArgs, (NG_DW(3, 2)), "dwconv_k3s2")
NG_KERNEL(KID_DW_K5S1, DwArgs, (NG_DW(5, 1)), "dwconv_k5s1")
NG_KERNEL(KID_DW_K5S2, DwArgs, (NG_DW(5, 2)), "dwconv_k5s2")
NG_KERNEL(KID_GAP, GapArgs, global_avgpool_tile, "global_avgpool")
NG_KERNEL(KID_FC_GEMV, FcArgs, fc_gemv_tile, "fc_gemv")
#define NG_PW(TM, TN, KC) conv1x1_mfma_tile<TM, TN, KC>
NG_KERNEL(KID_PW_32, PwArgs, (NG_PW(32, 32, 32)), "conv1x1_mfma_32x32")
NG_KERNEL(KID_PW_64, PwArgs, (NG_PW(64, 64, 16)), "conv1x1_mfma_64x64")
#define NG_C3(TP, S) conv3x3_tile<TP, S>
NG_KERNEL(KID_C3_T16S1, C3Args, (NG_C3(16, 1)), "conv3x3_t16s1")
NG_KERNEL(KID_C3_T16S2, C3Args, (NG_C3(16, 2)), "conv3x3_t16s2")
NG_KERNEL(KID_C3_T8S1, C3Args, (NG_C3(8, 1)), "conv3x3_t8s1")
NG_KERNEL(KID_C3_T8S2, C3Args, (NG_C3(8, 2)), "conv3x3_t8s2")

// Stand-alone kernel of one tile function: one workgroup per tile.
template <int KID>
__global__ __launch_bounds__(kBlock) void standalone_kernel(typename KernelOf<KID>::Args a) {
    __shared__ float smem[kSmemFloats];
    KernelOf<KID>::tile(a, blockIdx.x, smem);
}

// ------------------------------------------------------------------------------------
// Device-resident replay. The recorded schedule (Section 4.1: submission order, kernel
// arguments, task-to-stream assignment, synchronisations) sits in device memory and
// persistent workgroups execute it themselves, so a dependent task starts as soon as a
// counter in memory says its producers are done, instead of after a round trip through
// the command processor. Streams keep the meaning they have in Section 2 ("GPU Streams"):
// each stream is served, in FIFO order, by its own gang of workgroups (picked on one XCD,
// so a stream's tensors stay in that XCD's L2); an event is a completion counter:
// recording = each workgroup of the producer adds 1 with release semantics after its
// tiles, waiting = polling until the counter reaches (workgroups of the producer) x
// (replay number), then an acquire. Every wait is bounded: a workgroup that runs out of
// spins raises the error flag and every workgroup leaves.
// ------------------------------------------------------------------------------------
typedef const __attribute__((address_space(4))) DevTask* ConstTaskPtr;
typedef const __attribute__((address_space(4))) DevEntry* ConstEntryPtr;
typedef const __attribute__((address_space(4))) int* ConstIntPtr;

template <int KID>
__device__ __forceinline__ void run_tiles(ConstTaskPtr t, int tile, int step, int ntiles, float* smem) {
    using A = typename KernelOf<KID>::Args;
    static_assert(sizeof(A) % 4 == 0, "argument blocks are copied word by word");
    A a;                                                         // uniform address, read-only space: lands in SGPRs
    const __attribute__((address_space(4))) unsigned* src =
        reinterpret_cast<const __attribute__((address_space(4))) unsigned*>(t->args);
    unsigned* dst = reinterpret_cast<unsigned*>(&a);
#pragma unroll
    for (unsigned i = 0; i < sizeof(A) / 4; ++i) dst[i] = src[i];
    for (; tile < ntiles; tile += step) KernelOf<KID>::tile(a, tile, smem);
}

__global__ __launch_bounds__(kBlock) void resident_kernel(DevPlan plan, unsigned epoch) {
    __shared__ float smem[kSmemFloats];
    __shared__ int s_abort;
    const int lane = threadIdx.x;
    if (lane == 0) s_abort = 0;
    ConstTaskPtr tasks = (ConstTaskPtr)plan.tasks;
    ConstEntryPtr entries = (ConstEntryPtr)plan.entries;
    ConstIntPtr wg_first = (ConstIntPtr)plan.wg_first;
    const int e_begin = wg_first[blockIdx.x], e_end = wg_first[blockIdx.x + 1];
    __syncthreads();

    for (int e = e_begin; e < e_end; ++e) {
        const int task = entries[e].task, tile0 = entries[e].tile_begin, step = entries[e].tile_step;
        ConstTaskPtr t = tasks + task;
        const int np = t->n_parents;
        if (np > 0) {
            if (lane < 64) {                                    // first wavefront: lane j watches parent j
                bool ok = true;
                if (lane < np) {
                    const DevTask* tg = plan.tasks + task;      // per-lane index: ordinary loads
                    const unsigned target = tg->need[lane] * epoch;
                    const unsigned* counter = plan.done + tg->parent[lane];
                    unsigned spins = 0;
                    while ((int)(__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
                        if (++spins > plan.spin_limit ||
                            ((spins & 63u) == 0 && __hip_atomic_load(plan.error_dev, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                            ok = false;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(1);
                    }
                    if (!ok && spins > plan.spin_limit) {
                        atomicExch(plan.error_dev, task + 1);
                        *plan.error_host = task + 1;
                    }
                }
                if (__any(!ok)) {
                    if (lane == 0) s_abort = 1;
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // producers' data becomes visible to this CU
            }
            __syncthreads();
            if (s_abort) return;
        }
        switch (t->kid) {
#define NG_CASE(KID) case KID: run_tiles<KID>(t, tile0, step, t->ntiles, smem); break;
            NG_CASE(KID_BN) NG_CASE(KID_BN_V4) NG_CASE(KID_ADD) NG_CASE(KID_ADD_V4) NG_CASE(KID_CONCAT)
            NG_CASE(KID_CONCAT_V4) NG_CASE(KID_POOL) NG_CASE(KID_DW_K3S1) NG_CASE(KID_DW_K3S2)
            NG_CASE(KID_DW_K5S1) NG_CASE(KID_DW_K5S2) NG_CASE(KID_GAP) NG_CASE(KID_FC_GEMV)
            NG_CASE(KID_PW_32) NG_CASE(KID_PW_64) NG_CASE(KID_C3_T16S1) NG_CASE(KID_C3_T16S2)
            NG_CASE(KID_C3_T8S1) NG_CASE(KID_C3_T8S2)
#undef NG_CASE
            default: break;
        }
        __syncthreads();                                         // every thread's stores have been issued and counted
        if (lane == 0) __hip_atomic_fetch_add(plan.done + task, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ------------------------------------------------------------------------------------
// task construction
// ------------------------------------------------------------------------------------
template <int KID>
void set_kernel(Task& t, const typename KernelOf<KID>::Args& a, long ntiles) {
    using A = typename KernelOf<KID>::Args;
    static_assert(sizeof(A) <= kArgBytes, "argument block too large");
    static_assert(std::is_trivially_copyable<A>::value, "argument block must be plain data");
    t.kid = KID;
    t.fn = reinterpret_cast<const void*>(&standalone_kernel<KID>);
    t.name = KernelOf<KID>::name;
    std::memcpy(t.args, &a, sizeof(A));
    t.args_bytes = sizeof(A);
    t.ntiles = ntiles;
    t.grid[0] = (unsigned)ntiles;
}

long ceil_div(long a, long b) { return (a + b - 1) / b; }

}  // namespace

const void* resident_kernel_handle() { return reinterpret_cast<const void*>(&resident_kernel); }

int build_task(ng_graph* g, int v, char* arena, Task& t) {
    const Node& nd = g->nodes[v];
    t = Task();
    t.block[0] = kBlock;
    if (nd.op == NG_OP_INPUT) return NG_OK;
    for (size_t j = 0; j < nd.weights.size(); ++j)
        if (!nd.weights[j]) return g->fail(NG_EINVAL, "node %d: weight %d is a null device pointer", v, (int)j);

    auto buf = [&](int id) { return reinterpret_cast<float*>(arena + g->offset[id]); };
    const Shape& o = nd.out;
    const Shape& i0 = g->nodes[nd.preds[0]].out;
    const int total = (int)o.elems();
    const int hw_out = (int)(o.h * o.w);
    auto wf = [&](int j) { return static_cast<const float*>(nd.weights[j]); };

    switch (nd.op) {
        case NG_OP_BN_ACT:
        case NG_OP_RELU: {
            BnArgs a{};
            a.x = buf(nd.preds[0]);
            a.y = buf(v);
            if (nd.op == NG_OP_BN_ACT) {
                a.gamma = wf(0), a.beta = wf(1), a.mean = wf(2), a.var = wf(3);
                a.eps = nd.p.eps;
                a.relu = nd.p.relu != 0;
            } else {
                a.relu = 1;
            }
            a.C = (int)o.c, a.HW = hw_out, a.total = total;
            if (hw_out % 4 == 0) set_kernel<KID_BN_V4>(t, a, ceil_div(total / 4, kBlock));
            else set_kernel<KID_BN>(t, a, ceil_div(total, kBlock));
            break;
        }
        case NG_OP_ADD_N: {
            AddArgs a{};
            a.k = (int)nd.preds.size();
            for (int j = 0; j < NG_MAX_PREDS; ++j) a.x[j] = buf(nd.preds[j < a.k ? j : 0]);
            a.y = buf(v);
            a.total = total;
            if (total % 4 == 0) set_kernel<KID_ADD_V4>(t, a, ceil_div(total / 4, kBlock));
            else set_kernel<KID_ADD>(t, a, ceil_div(total, kBlock));
            break;
        }
        case NG_OP_CONCAT: {
            ConcatArgs a{};
            a.k = (int)nd.preds.size();
            int first = 0;
            for (int j = 0; j < a.k; ++j) {
                a.x[j] = buf(nd.preds[j]);
                a.cin[j] = (int)g->nodes[nd.preds[j]].out.c;
                a.lo[j] = nd.p.slice_lo[j];
                a.first[j] = first;
                first += nd.p.slice_hi[j] - nd.p.slice_lo[j];
            }
            for (int j = a.k; j < NG_MAX_PREDS; ++j) a.x[j] = a.x[0], a.first[j] = first;
            a.y = buf(v);
            a.C = (int)o.c, a.HW = hw_out, a.total = total;
            if (hw_out % 4 == 0) set_kernel<KID_CONCAT_V4>(t, a, ceil_div(total / 4, kBlock));
            else set_kernel<KID_CONCAT>(t, a, ceil_div(total, kBlock));
            break;
        }
        case NG_OP_POOL: {
            PoolArgs a{buf(nd.preds[0]), buf(v), (int)i0.h, (int)i0.w, (int)o.h, (int)o.w,
                       nd.p.stride, nd.p.pad, nd.p.pool_mode, total};
            set_kernel<KID_POOL>(t, a, ceil_div(total, kBlock));
            break;
        }
        case NG_OP_DWCONV: {
            DwArgs a{buf(nd.preds[0]), wf(0), buf(v), (int)o.c, (int)i0.h, (int)i0.w, (int)o.h, (int)o.w, total};
            const long n = ceil_div(total, kBlock);
            if (nd.p.k == 3 && nd.p.stride == 1) set_kernel<KID_DW_K3S1>(t, a, n);
            else if (nd.p.k == 3) set_kernel<KID_DW_K3S2>(t, a, n);
            else if (nd.p.stride == 1) set_kernel<KID_DW_K5S1>(t, a, n);
            else set_kernel<KID_DW_K5S2>(t, a, n);
            break;
        }
        case NG_OP_GLOBAL_AVGPOOL: {
            GapArgs a{buf(nd.preds[0]), buf(v), (int)(i0.h * i0.w), (int)(o.n * o.c)};
            set_kernel<KID_GAP>(t, a, ceil_div(a.planes, kBlock / 64));
            break;
        }
        case NG_OP_FC:
        case NG_OP_CONV1X1: {
            const bool fc = nd.op == NG_OP_FC;
            if (fc && o.n <= 8) {
                FcArgs a{buf(nd.preds[0]), wf(0), wf(1), buf(v), (int)o.n, (int)i0.c, (int)o.c};
                set_kernel<KID_FC_GEMV>(t, a, ceil_div(a.Cout, kBlock / 64));
                break;
            }
            PwArgs a{buf(nd.preds[0]), wf(0), fc ? wf(1) : nullptr, buf(v), (int)i0.c, (int)o.c, hw_out,
                     (int)(o.n * hw_out), 0};
            const long big_tiles = ceil_div(a.Cout, 64) * ceil_div(a.cols, 64);
            if (big_tiles >= 256) {
                a.tiles_n = (int)ceil_div(a.cols, 64);
                set_kernel<KID_PW_64>(t, a, big_tiles);
            } else {
                a.tiles_n = (int)ceil_div(a.cols, 32);
                set_kernel<KID_PW_32>(t, a, (long)a.tiles_n * ceil_div(a.Cout, 32));
            }
            break;
        }
        case NG_OP_CONV3X3: {
            C3Args a{buf(nd.preds[0]), wf(0), buf(v), (int)i0.c, (int)o.c, (int)i0.h, (int)i0.w,
                     (int)o.h, (int)o.w, nd.p.pad, 0, 0, 0};
            const bool small = o.h * o.w <= 24 * 24;       // small maps: 8 x 8 tiles waste fewer lanes
            const int tp = small ? 8 : 16;
            a.tiles_x = (int)ceil_div(o.w, tp);
            a.tiles_xy = a.tiles_x * (int)ceil_div(o.h, tp);
            a.co_groups = (int)ceil_div(a.Cout, small ? 32 : 8);
            const long n = (long)a.tiles_xy * a.co_groups * o.n;
            if (small) {
                if (nd.p.stride == 1) set_kernel<KID_C3_T8S1>(t, a, n); else set_kernel<KID_C3_T8S2>(t, a, n);
            } else {
                if (nd.p.stride == 1) set_kernel<KID_C3_T16S1>(t, a, n); else set_kernel<KID_C3_T16S2>(t, a, n);
            }
            break;
        }
        default:
            return g->fail(NG_EINVAL, "node %d: operator %d has no kernel", v, nd.op);
    }
    if (t.ntiles <= 0 || t.ntiles >= (1L << 31)) return g->fail(NG_ESHAPE, "node %d: %ld tiles cannot be launched", v, t.ntiles);
    return NG_OK;
}

}  // namespace ng
