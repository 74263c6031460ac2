// GPU tasks of the AoT multi-stream DAG executor: fp32 NCHW kernels for gfx950 (wave64).
//
// The Nimble paper (arXiv 2012.02732) ships no kernels of its own: it replays the base
// framework's operators unchanged (Section 5, "Experimental Setup"). These are the
// operators of its benchmark networks, written for CDNA4. Each kernel takes ONE by-value
// argument struct so that the task table can hold a ready-made argument block per task
// (Section 4.1: kernel arguments are prepared once, ahead of time).
//
// Sizing rule that differs from usual throughput tuning: tasks are small (tens of
// thousands of elements) and are meant to run next to sibling tasks of other streams
// (Section 2, "GPU Streams"), so grids are sized by the work, never "fill the chip".
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>

#include "ng_internal.h"

namespace ng {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;

// ------------------------------------------------------------------------------------
// bn_act / relu: y = x * s[c] + t[c] (s, t folded from gamma, beta, mean, var), optional ReLU
// ------------------------------------------------------------------------------------
struct BnArgs {
    const float* x;
    float* y;
    const float* gamma;   // nullptr => plain ReLU
    const float* beta;
    const float* mean;
    const float* var;
    float eps;
    int relu;
    int C, HW;
    int total;            // elements
};

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
__global__ __launch_bounds__(kBlock) void bn_act_kernel(BnArgs a) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
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
struct AddArgs {
    const float* x[NG_MAX_PREDS];
    float* y;
    int k;
    int total;
};

template <bool VEC4>
__global__ __launch_bounds__(kBlock) void add_n_kernel(AddArgs a) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (VEC4) {
        const int e = i * 4;
        if (e >= a.total) return;
        float4 acc = *reinterpret_cast<const float4*>(a.x[0] + e);
        for (int j = 1; j < a.k; ++j) {
            const float4 v = *reinterpret_cast<const float4*>(a.x[j] + e);
            acc.x += v.x, acc.y += v.y, acc.z += v.z, acc.w += v.w;
        }
        *reinterpret_cast<float4*>(a.y + e) = acc;
    } else {
        if (i >= a.total) return;
        float acc = a.x[0][i];
        for (int j = 1; j < a.k; ++j) acc += a.x[j][i];
        a.y[i] = acc;
    }
}

// ------------------------------------------------------------------------------------
// concat: output channel block j = channels [lo_j, lo_j + cnt_j) of input j
// ------------------------------------------------------------------------------------
struct ConcatArgs {
    const float* x[NG_MAX_PREDS];
    float* y;
    int cin[NG_MAX_PREDS];     // channel count of input j
    int lo[NG_MAX_PREDS];      // first channel taken from input j
    int first[NG_MAX_PREDS];   // first output channel of block j
    int k;
    int C, HW;                 // output channels, pixels per plane
    int total;
};

template <bool VEC4>
__global__ __launch_bounds__(kBlock) void concat_kernel(ConcatArgs a) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
    const int e = VEC4 ? i * 4 : i;
    if (e >= a.total) return;
    const int plane = e / a.HW, pix = e - plane * a.HW;
    const int n = plane / a.C, c = plane - n * a.C;
    int j = 0;
    for (int q = 1; q < a.k; ++q)
        if (c >= a.first[q]) j = q;
    const float* src = a.x[j] + ((size_t)(n * a.cin[j] + a.lo[j] + c - a.first[j])) * a.HW + pix;
    if (VEC4)
        *reinterpret_cast<float4*>(a.y + e) = *reinterpret_cast<const float4*>(src);
    else
        a.y[e] = *src;
}

// ------------------------------------------------------------------------------------
// pool3x3: max (out-of-bounds taps ignored) or average over the in-bounds taps
// ------------------------------------------------------------------------------------
struct PoolArgs {
    const float* x;
    float* y;
    int H, W, Ho, Wo;
    int stride, pad, mode;     // mode 0 max, 1 avg
    int total;                 // output elements
};

__global__ __launch_bounds__(kBlock) void pool3x3_kernel(PoolArgs a) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
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
struct DwArgs {
    const float* x;
    const float* w;            // [C][K][K]
    float* y;
    int C, H, W, Ho, Wo;
    int total;                 // output elements
};

template <int K, int S>
__global__ __launch_bounds__(kBlock) void dwconv_kernel(DwArgs a) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
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
struct GapArgs {
    const float* x;
    float* y;
    int HW, planes;
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

__global__ __launch_bounds__(kBlock) void global_avgpool_kernel(GapArgs a) {
    const int lane = threadIdx.x & 63;
    const int plane = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
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
struct FcArgs {
    const float* x;            // [N][Cin]
    const float* w;            // [Cout][Cin]
    const float* b;            // [Cout]
    float* y;                  // [N][Cout]
    int N, Cin, Cout;
};

__global__ __launch_bounds__(kBlock) void fc_gemv_kernel(FcArgs a) {
    const int lane = threadIdx.x & 63;
    const int o = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
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
struct PwArgs {
    const float* x;            // [N][Cin][HW]
    const float* w;            // [Cout][Cin]
    const float* bias;         // [Cout] or nullptr
    float* y;                  // [N][Cout][HW]
    int Cin, Cout, HW, cols;
};

template <int TM, int TN, int KC>
__global__ __launch_bounds__(kBlock) void conv1x1_mfma_kernel(PwArgs a) {
    constexpr int WM = TM / 2, WN = TN / 2;           // per-wavefront sub-tile
    constexpr int FM = WM / 16, FN = WN / 16;         // 16 x 16 fragments per wavefront
    __shared__ float As[KC][TM + 1];
    __shared__ float Bs[KC][TN + 1];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;

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
            As[k][m] = (gm < a.Cout && gk < a.Cin) ? a.w[(size_t)gm * a.Cin + gk] : 0.f;
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
            Bs[k][n] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < KC; kk += 4) {
            float af[FM], bf[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) af[i] = As[kk + (lane >> 4)][wm * WM + i * 16 + (lane & 15)];
#pragma unroll
            for (int j = 0; j < FN; ++j) bf[j] = Bs[kk + (lane >> 4)][wn * WN + j * 16 + (lane & 15)];
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
// ------------------------------------------------------------------------------------
struct C3Args {
    const float* x;            // [N][Cin][H][W]
    const float* w;            // [Cout][Cin][3][3]
    float* y;                  // [N][Cout][Ho][Wo]
    int Cin, Cout, H, W, Ho, Wo;
    int pad;
    int tiles_x;               // pixel tiles along W
};

template <int TP, int S>
__global__ __launch_bounds__(kBlock) void conv3x3_kernel(C3Args a) {
    constexpr int CIC = 4;                             // input channels per LDS slice
    constexpr int IW = (TP - 1) * S + 3;               // input patch edge
    constexpr int GROUPS = TP == 16 ? 1 : 4;           // channel groups per workgroup
    constexpr int CO = 8;
    __shared__ float patch[CIC][IW][IW + 1];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int local = TP == 16 ? tid : (tid & 63);
    const int ty = local / TP, tx = local % TP;
    const int tile = blockIdx.x, tile_y = tile / a.tiles_x, tile_x = tile - tile_y * a.tiles_x;
    const int oy = tile_y * TP + ty, ox = tile_x * TP + tx;
    const int co0 = (blockIdx.y * GROUPS + (TP == 16 ? 0 : wave)) * CO;
    const int img = blockIdx.z;
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
            patch[ci][cy][cx] = v;
        }
        __syncthreads();
        const int nci = min(CIC, a.Cin - c0);
        for (int ci = 0; ci < nci; ++ci) {
            float in[9];
#pragma unroll
            for (int dr = 0; dr < 3; ++dr)
#pragma unroll
                for (int dc = 0; dc < 3; ++dc) in[dr * 3 + dc] = patch[ci][ty * S + dr][tx * S + dc];
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
// task construction
// ------------------------------------------------------------------------------------
template <class A>
void put_args(Task& t, const A& a) {
    static_assert(sizeof(A) <= sizeof(t.args), "argument block too large");
    static_assert(std::is_trivially_copyable<A>::value, "argument block must be plain data");
    std::memcpy(t.args, &a, sizeof(A));
    t.args_bytes = sizeof(A);
}

unsigned blocks_for(long items) { return (unsigned)((items + kBlock - 1) / kBlock); }

template <class F>
void set_fn(Task& t, F* fn, const char* name) {
    t.fn = reinterpret_cast<const void*>(fn);
    t.name = name;
}

}  // namespace

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
            const bool vec = hw_out % 4 == 0;
            if (vec) set_fn(t, &bn_act_kernel<true>, "bn_act_v4"); else set_fn(t, &bn_act_kernel<false>, "bn_act");
            t.grid[0] = blocks_for(vec ? total / 4 : total);
            put_args(t, a);
            break;
        }
        case NG_OP_ADD_N: {
            AddArgs a{};
            a.k = (int)nd.preds.size();
            for (int j = 0; j < a.k; ++j) a.x[j] = buf(nd.preds[j]);
            a.y = buf(v);
            a.total = total;
            const bool vec = total % 4 == 0;
            if (vec) set_fn(t, &add_n_kernel<true>, "add_n_v4"); else set_fn(t, &add_n_kernel<false>, "add_n");
            t.grid[0] = blocks_for(vec ? total / 4 : total);
            put_args(t, a);
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
            a.y = buf(v);
            a.C = (int)o.c, a.HW = hw_out, a.total = total;
            const bool vec = hw_out % 4 == 0;
            if (vec) set_fn(t, &concat_kernel<true>, "concat_v4"); else set_fn(t, &concat_kernel<false>, "concat");
            t.grid[0] = blocks_for(vec ? total / 4 : total);
            put_args(t, a);
            break;
        }
        case NG_OP_POOL: {
            PoolArgs a{buf(nd.preds[0]), buf(v), (int)i0.h, (int)i0.w, (int)o.h, (int)o.w,
                       nd.p.stride, nd.p.pad, nd.p.pool_mode, total};
            set_fn(t, &pool3x3_kernel, "pool3x3");
            t.grid[0] = blocks_for(total);
            put_args(t, a);
            break;
        }
        case NG_OP_DWCONV: {
            DwArgs a{buf(nd.preds[0]), wf(0), buf(v), (int)o.c, (int)i0.h, (int)i0.w, (int)o.h, (int)o.w, total};
            if (nd.p.k == 3 && nd.p.stride == 1) set_fn(t, &dwconv_kernel<3, 1>, "dwconv_k3s1");
            else if (nd.p.k == 3) set_fn(t, &dwconv_kernel<3, 2>, "dwconv_k3s2");
            else if (nd.p.stride == 1) set_fn(t, &dwconv_kernel<5, 1>, "dwconv_k5s1");
            else set_fn(t, &dwconv_kernel<5, 2>, "dwconv_k5s2");
            t.grid[0] = blocks_for(total);
            put_args(t, a);
            break;
        }
        case NG_OP_GLOBAL_AVGPOOL: {
            GapArgs a{buf(nd.preds[0]), buf(v), (int)(i0.h * i0.w), (int)(o.n * o.c)};
            set_fn(t, &global_avgpool_kernel, "global_avgpool");
            t.grid[0] = (unsigned)((a.planes + 3) / 4);
            put_args(t, a);
            break;
        }
        case NG_OP_FC:
        case NG_OP_CONV1X1: {
            const bool fc = nd.op == NG_OP_FC;
            if (fc && o.n <= 8) {
                FcArgs a{buf(nd.preds[0]), wf(0), wf(1), buf(v), (int)o.n, (int)i0.c, (int)o.c};
                set_fn(t, &fc_gemv_kernel, "fc_gemv");
                t.grid[0] = (unsigned)((a.Cout + 3) / 4);
                put_args(t, a);
                break;
            }
            PwArgs a{buf(nd.preds[0]), wf(0), fc ? wf(1) : nullptr, buf(v), (int)i0.c, (int)o.c, hw_out,
                     (int)(o.n * hw_out)};
            const long big_tiles = ((a.Cout + 63) / 64) * (long)((a.cols + 63) / 64);
            if (big_tiles >= 256) {
                set_fn(t, &conv1x1_mfma_kernel<64, 64, 16>, "conv1x1_mfma_64x64");
                t.grid[0] = (unsigned)((a.cols + 63) / 64), t.grid[1] = (unsigned)((a.Cout + 63) / 64);
            } else {
                set_fn(t, &conv1x1_mfma_kernel<32, 32, 32>, "conv1x1_mfma_32x32");
                t.grid[0] = (unsigned)((a.cols + 31) / 32), t.grid[1] = (unsigned)((a.Cout + 31) / 32);
            }
            put_args(t, a);
            break;
        }
        case NG_OP_CONV3X3: {
            C3Args a{buf(nd.preds[0]), wf(0), buf(v), (int)i0.c, (int)o.c, (int)i0.h, (int)i0.w,
                     (int)o.h, (int)o.w, nd.p.pad, 0};
            const bool small = o.h * o.w <= 24 * 24;       // small maps: 8 x 8 tiles waste fewer lanes
            const int tp = small ? 8 : 16;
            a.tiles_x = (int)((o.w + tp - 1) / tp);
            const int tiles_y = (int)((o.h + tp - 1) / tp);
            const int per_wg = small ? 32 : 8;            // output channels per workgroup
            if (small) {
                if (nd.p.stride == 1) set_fn(t, &conv3x3_kernel<8, 1>, "conv3x3_t8s1");
                else set_fn(t, &conv3x3_kernel<8, 2>, "conv3x3_t8s2");
            } else {
                if (nd.p.stride == 1) set_fn(t, &conv3x3_kernel<16, 1>, "conv3x3_t16s1");
                else set_fn(t, &conv3x3_kernel<16, 2>, "conv3x3_t16s2");
            }
            t.grid[0] = (unsigned)(a.tiles_x * tiles_y);
            t.grid[1] = (unsigned)((a.Cout + per_wg - 1) / per_wg);
            t.grid[2] = (unsigned)o.n;
            put_args(t, a);
            break;
        }
        default:
            return g->fail(NG_EINVAL, "node %d: operator %d has no kernel", v, nd.op);
    }
    if (t.grid[1] > 65535 || t.grid[2] > 65535) return g->fail(NG_ESHAPE, "node %d: launch grid too large", v);
    return NG_OK;
}

}  // namespace ng
