// GPU tasks of the AoT multi-stream DAG executor: fp32 NCHW kernels for gfx950 (wave64).
//
// The Nimble paper (arXiv 2012.02732) ships no kernels of its own: it replays the base
// framework's operators unchanged (Section 5, "Experimental Setup"). These are the
// operators of its benchmark networks, written for CDNA4.
//
// Every operator is written once as a *tile function*: the share of 256 threads,
// addressed by a linear tile index. Two kinds of kernels are built from them:
//   * one stand-alone kernel per tile function (grid = number of tiles, 256 threads),
//     taking ONE by-value argument struct so that the task table can hold a ready-made
//     argument block per task (Section 4.1: kernel arguments are prepared once, ahead of time);
//   * the device-resident replay kernel at the end of this file, in which persistent
//     workgroups of 512 threads (two tiles at a time) walk the recorded task schedule
//     themselves.
//
// Sizing rule that differs from usual throughput tuning: tasks are small (tens of
// thousands of elements) and are meant to run next to sibling tasks of other streams
// (Section 2, "GPU Streams"), so grids are sized by the work, never "fill the chip".
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <type_traits>

#include "ng_device.h"
#include "ng_internal.h"

namespace ng {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Access helpers. `far` is a compile-time constant at every call site. A far access is a
// device-scope access (sc1): it is served by the memory side, past the XCD-private L2, which
// is what makes a tensor written on one XCD readable on another without flushing or
// invalidating either L2. Far accesses go through buffer instructions (uniform tensor base
// + 32-bit byte offset), which carry the cache policy and come in 128-bit form; tensors are
// far smaller than the 4 GiB a 32-bit offset spans.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr int kPolicyDeviceScope = 16;                       // cache-policy operand: sc1

__device__ __forceinline__ __amdgpu_buffer_rsrc_t tensor_rsrc(const float* base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, 0x7FFFFFFF, 0x00020000);
}
__device__ __forceinline__ unsigned byte_offset(const float* base, const float* p) {
    return (unsigned)(reinterpret_cast<const char*>(p) - reinterpret_cast<const char*>(base));
}
// base: wave-uniform start of the tensor; p: this lane's address inside it
__device__ __forceinline__ float ldg(const float* base, const float* p, bool far) {
    if (!far) return *p;
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(tensor_rsrc(base), byte_offset(base, p), 0, kPolicyDeviceScope));
}
__device__ __forceinline__ float4 ldg4(const float* base, const float* p, bool far) {
    if (!far) return *reinterpret_cast<const float4*>(p);
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(tensor_rsrc(base), byte_offset(base, p), 0, kPolicyDeviceScope);
    float4 f;
    __builtin_memcpy(&f, &v, sizeof f);                     // the whole vector at once: extracting elements one by
    return f;                                               // one makes this compiler shrink the load to one dword
}
__device__ __forceinline__ void stg(float* base, float* p, float v, bool far) {
    if (!far) {
        *p = v;
        return;
    }
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), tensor_rsrc(base), byte_offset(base, p), 0, kPolicyDeviceScope);
}
__device__ __forceinline__ void stg4(float* base, float* p, float4 v, bool far) {
    if (!far) {
        *reinterpret_cast<float4*>(p) = v;
        return;
    }
    u32x4 u;
    __builtin_memcpy(&u, &v, sizeof u);
    __builtin_amdgcn_raw_buffer_store_b128(u, tensor_rsrc(base), byte_offset(base, p), 0, kPolicyDeviceScope);
}
// per-lane tensor (concat picks its source per lane): single relaxed device-scope accesses
__device__ __forceinline__ float ldg_any(const float* p, bool far) {
    return far ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *p;
}
// 128-bit device-scope load from a per-lane address (16-byte aligned). The compiler does not
// know about loads issued from inline assembly, so the wait for the data is part of it.
__device__ __forceinline__ float4 ldg4_any_far(const float* p) {
    f32x4 v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
    return make_float4(v[0], v[1], v[2], v[3]);
}

// LDS floats every workgroup owns: the largest users are the conv3x3 input patches (4 x 33 x 34; 256 pixels x 20).
constexpr int kSmemFloats = 5120;
// ... and what the conv3x3 kernels with a patch of up to 640 pixels get instead (stand-alone kernels: only they; the
// resident kernel: every workgroup of the build that contains them)
constexpr int kSmemFloatsWide = 12800;
constexpr bool has_wide_patch(int kid) { return kid == KID_C3_Q32 || kid == KID_C3_Q64 || kid == KID_C3_Q128; }
constexpr int smem_floats(int kid) { return has_wide_patch(kid) ? kSmemFloatsWide : kSmemFloats; }

// ------------------------------------------------------------------------------------
// bn_act / relu: y = x * s[c] + t[c] (s, t folded from gamma, beta, mean, var), optional ReLU
// ------------------------------------------------------------------------------------
__device__ __forceinline__ void bn_coeff(const BnArgs& a, int c, float& s, float& t) {
    if (a.scale) {
        s = a.scale[c];
        t = a.shift[c];
    } else {
        s = 1.f;
        t = 0.f;
    }
}

// Batch-norm parameters -> one multiplier and one offset per channel, once, at bind time.
__global__ __launch_bounds__(kBlock) void fold_bn_kernel(const float* gamma, const float* beta, const float* mean,
                                                         const float* var, float eps, float* scale, float* shift, int C) {
    const int c = blockIdx.x * kBlock + threadIdx.x;
    if (c >= C) return;
    const float s = gamma[c] / sqrtf(var[c] + eps);
    scale[c] = s;
    shift[c] = beta[c] - mean[c] * s;
}

// Every tile function takes a `wait` object and calls it exactly once, on every path and by
// every thread of the workgroup (it may contain a workgroup barrier), before the first access
// to data another task produced. Whatever does not depend on such data - index arithmetic,
// reading weights and coefficients - goes before the call, so that it overlaps with waiting
// for the producers. Stand-alone kernels pass NoWait; the resident kernel passes the wait
// for the task's completion counters, which does its work on the first call only.
// A convolution tile with a fused add_n calls `late` the same way, once, before it reads the
// other operands of the sum.
// A tile function meets the same number of workgroup barriers whatever its tile index and whether
// or not it is `live`: in the resident kernel two sub-blocks of one workgroup run different tiles
// of a task side by side and share every barrier.
struct NoWait {
    __device__ __forceinline__ void operator()() const {}
    __device__ __forceinline__ void late() const {}
    __device__ __forceinline__ constexpr bool far_out() const { return false; }
};

// Store one convolution result and, if a batch-norm / ReLU task was fused into the tile, that
// task's result as well (the kernels for larger problems: coefficients are fetched here, per
// value; the 16-row kernels fetch theirs before they wait for their inputs).
__device__ __forceinline__ void store_with_epilogue(float* y, const Epilogue& ep, size_t at, int channel, float v, bool fout) {
    stg(y, y + at, v, fout);
    if (ep.y != nullptr) {
        float s = 1.f, t = 0.f;
        if (ep.scale != nullptr) s = ep.scale[channel], t = ep.shift[channel];
        const float z = fmaf(v, s, t);
        stg(ep.y, ep.y + at, ep.relu ? fmaxf(z, 0.f) : z, fout);
    }
}

// The add_n epilogue of a convolution tile: v holds this lane's values (4 consecutive pixels if
// VEC, else one), `at` their position in the tensors; the sum runs in argument order.
template <bool VEC>
__device__ __forceinline__ void add_epilogue(const AddEpilogue& ea, float4 v, size_t at, bool fout) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int j = 0; j < kEpilogueAddMax; ++j) {               // constant indices only: the argument block stays in scalar registers
        if (j >= ea.k) break;
        float4 t = v;
        if (j != ea.zpos) {
            const float* x = j > ea.zpos ? ea.x[j > 0 ? j - 1 : 0] : ea.x[j < kEpilogueAddMax - 1 ? j : kEpilogueAddMax - 2];
            if (VEC) t = ldg4(x, x + at, ea.far != 0);
            else t.x = ldg(x, x + at, ea.far != 0);
        }
        if (j == 0) acc = t;
        else acc.x += t.x, acc.y += t.y, acc.z += t.z, acc.w += t.w;
    }
    if (VEC) stg4(ea.y, ea.y + at, acc, fout);
    else stg(ea.y, ea.y + at, acc.x, fout);
}

// Elementwise operators come in four partitions of the output into tiles, so that an
// elementwise task can take over the partition of the task that feeds it (then tile i of
// the consumer reads only what tile i of the producer wrote, and a workgroup that ran the
// one can run the other without waiting for anybody else):
//   PART_L256  tile t = elements [256 t, 256 t + 256), one per thread (pool, dwconv order)
//   PART_L1024 tile t = elements [1024 t, 1024 t + 1024), one float4 per thread
//   PART_R64   tile t = 16 channels x 64 columns (column = image * HW + pixel), the tile of
//              the 128-bit conv1x1; thread = (channel tid / 16, 4 columns from 4 (tid % 16))
//   PART_R16   tile t = 16 channels x 16 columns, the tile of the 32-bit conv1x1
// ElemIndex: first element a thread owns (VEC of them, consecutive), its channel, validity.
struct ElemIndex {
    int e, c;
    bool ok;
};
template <int PART>
__device__ __forceinline__ ElemIndex elem_index(int tile, int tid, int C, int HW, int total, int cols) {
    ElemIndex r;
    if (PART == PART_L1024 || PART == PART_L256) {
        r.e = (tile * kBlock + tid) * (PART == PART_L1024 ? 4 : 1);
        r.ok = r.e < total;
        r.c = (r.e / HW) % C;
    } else {
        constexpr int TN = PART == PART_R64 ? 64 : 16, V = PART == PART_R64 ? 4 : 1;
        const int tiles_n = (cols + TN - 1) / TN;
        const int by = tile / tiles_n, bx = tile - by * tiles_n;
        const int col = bx * TN + V * (tid & 15);
        r.c = by * 16 + (tid >> 4);
        r.ok = r.c < C && col < cols;
        const int img = col / HW, pix = col - img * HW;
        r.e = (img * C + r.c) * HW + pix;
    }
    return r;
}

template <int PART, bool FIN, class Wait>
__device__ __forceinline__ void bn_act_tile(const BnArgs& a, int tile, float*, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    const ElemIndex ix = elem_index<PART>(tile, tid, a.C, a.HW, a.total, a.cols);
    const bool active = live && ix.ok;
    float s = 1.f, t = 0.f;
    if (active) bn_coeff(a, ix.c, s, t);
    wait();
    if (!active) return;
    if (PART == PART_L1024 || PART == PART_R64) {          // HW % 4 == 0: a float4 never straddles channels
        float4 v = ldg4(a.x, a.x + ix.e, FIN);
        v.x = fmaf(v.x, s, t), v.y = fmaf(v.y, s, t), v.z = fmaf(v.z, s, t), v.w = fmaf(v.w, s, t);
        if (a.relu) v.x = fmaxf(v.x, 0.f), v.y = fmaxf(v.y, 0.f), v.z = fmaxf(v.z, 0.f), v.w = fmaxf(v.w, 0.f);
        stg4(a.y, a.y + ix.e, v, fout);
    } else {
        const float v = fmaf(ldg(a.x, a.x + ix.e, FIN), s, t);
        stg(a.y, a.y + ix.e, a.relu ? fmaxf(v, 0.f) : v, fout);
    }
}

// ------------------------------------------------------------------------------------
// add_n: elementwise sum of k tensors, accumulated in argument order
// ------------------------------------------------------------------------------------
template <int PART, bool FIN, class Wait>
__device__ __forceinline__ void add_n_tile(const AddArgs& a, int tile, float*, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    const ElemIndex ix = elem_index<PART>(tile, tid, a.C, a.HW, a.total, a.cols);
    wait();
    if (!live || !ix.ok) return;
    const int e = ix.e;
    if (PART == PART_L1024 || PART == PART_R64) {
        float4 acc = ldg4(a.x[0], a.x[0] + e, FIN);
#pragma unroll
        for (int j = 1; j < NG_MAX_PREDS; ++j) {
            if (j >= a.k) break;
            const float4 v = ldg4(a.x[j], a.x[j] + e, FIN);
            acc.x += v.x, acc.y += v.y, acc.z += v.z, acc.w += v.w;
        }
        stg4(a.y, a.y + e, acc, fout);
    } else {
        float acc = ldg(a.x[0], a.x[0] + e, FIN);
#pragma unroll
        for (int j = 1; j < NG_MAX_PREDS; ++j) {
            if (j >= a.k) break;
            acc += ldg(a.x[j], a.x[j] + e, FIN);
        }
        stg(a.y, a.y + e, acc, fout);
    }
}

// ------------------------------------------------------------------------------------
// concat: output channel block j = channels [lo_j, lo_j + cnt_j) of input j
// ------------------------------------------------------------------------------------
template <bool VEC4, bool FIN, class Wait>
__device__ __forceinline__ void concat_tile(const ConcatArgs& a, int tile, float*, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    const int i = tile * kBlock + tid;
    const int e = VEC4 ? i * 4 : i;
    const bool active = live && e < a.total;
    const int plane = e / a.HW, pix = e - plane * a.HW;
    const int n = plane / a.C, c = plane - n * a.C;
    const float* base = a.x[0];
    int cin = a.cin[0], lo = a.lo[0], first = a.first[0];
#pragma unroll
    for (int q = 1; q < NG_MAX_PREDS; ++q)
        if (q < a.k && c >= a.first[q]) base = a.x[q], cin = a.cin[q], lo = a.lo[q], first = a.first[q];
    const float* src = base + ((size_t)(n * cin + lo + c - first)) * a.HW + pix;
    wait();
    if (!active || src == a.y + e) return;                   // an input the memory plan placed inside the result is there already
    if (VEC4) {
        float4 v;
        if (FIN) v = ldg4_any_far(src);
        else v = *reinterpret_cast<const float4*>(src);
        stg4(a.y, a.y + e, v, fout);
    } else {
        stg(a.y, a.y + e, ldg_any(src, FIN), fout);
    }
}

// ------------------------------------------------------------------------------------
// pool3x3: max (out-of-bounds taps ignored) or average over the in-bounds taps
// ------------------------------------------------------------------------------------
// Windowed kernels: a tile is 256 P consecutive outputs, thread t owns outputs t, t + 256, ...
// of it (P = 1 for stand-alone launches; P = 4 when a task would otherwise need several
// rounds on the workgroups of its stream - one round costs one trip to memory however many
// loads are in flight, and 1024 consecutive outputs are also the tile of the float4
// elementwise kernels, which can then take over the partition).
template <int P, bool EA, bool FIN, class Wait>
__device__ __forceinline__ void pool3x3_tile(const typename std::conditional<EA, PoolAddArgs, PoolArgs>::type& a, int tile, float*, int tid,
                                             bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    const int base = tile * kBlock * P + tid;
    const bool active = live && base < a.total;
    // all taps of all P outputs are loaded unconditionally from clamped coordinates, so the
    // loads are independent and in flight together; taps outside the image are masked afterwards
    float v[P][9];
    int r0[P], c0[P];
    const float* src[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int i = min(base + p * kBlock, a.total - 1);
        const int ow = i % a.Wo, t = i / a.Wo;
        const int oh = t % a.Ho, plane = t / a.Ho;
        src[p] = a.x + (size_t)plane * a.H * a.W;
        r0[p] = oh * a.stride - a.pad, c0[p] = ow * a.stride - a.pad;
    }
    wait();
    if (!EA && !active) return;                              // with a fused add_n every thread goes on to the late wait
    float res[P];
    if (active) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
#pragma unroll
            for (int dr = 0; dr < 3; ++dr)
#pragma unroll
                for (int dc = 0; dc < 3; ++dc)
                    v[p][dr * 3 + dc] = ldg(a.x, src[p] + min(max(r0[p] + dr, 0), a.H - 1) * a.W + min(max(c0[p] + dc, 0), a.W - 1), FIN);
        }
        __builtin_amdgcn_sched_barrier(0);                   // all loads are issued before the first use
#pragma unroll
        for (int p = 0; p < P; ++p) {
            float acc = a.mode == 0 ? -INFINITY : 0.f;
            int cnt = 0;
#pragma unroll
            for (int dr = 0; dr < 3; ++dr)
#pragma unroll
                for (int dc = 0; dc < 3; ++dc) {
                    const int r = r0[p] + dr, c = c0[p] + dc;
                    const bool in = r >= 0 && r < a.H && c >= 0 && c < a.W;
                    if (a.mode == 0) acc = in ? fmaxf(acc, v[p][dr * 3 + dc]) : acc;
                    else acc += in ? v[p][dr * 3 + dc] : 0.f;
                    cnt += in;
                }
            res[p] = a.mode == 0 ? acc : acc / (float)cnt;
            if (base + p * kBlock < a.total) stg(a.y, a.y + base + p * kBlock, res[p], fout);
        }
    }
    if constexpr (EA) {
        wait.late();
        if (active) {
#pragma unroll
            for (int p = 0; p < P; ++p)
                if (base + p * kBlock < a.total)
                    add_epilogue<false>(a.ea, make_float4(res[p], 0.f, 0.f, 0.f), (size_t)(base + p * kBlock), fout);
        }
    }
}

// ------------------------------------------------------------------------------------
// dwconv: depthwise K x K, pad K/2, stride S; P outputs per thread
// ------------------------------------------------------------------------------------
template <int K, int S, int P, bool FIN, class Wait>
__device__ __forceinline__ void dwconv_tile(const DwArgs& a, int tile, float*, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    const int base = tile * kBlock * P + tid;
    const bool active = live && base < a.total;
    // unconditional loads from clamped coordinates (all in flight together), masked afterwards
    float v[P][K * K], w[P][K * K];
    int r0[P], c0[P];
    const float* src[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int i = min(base + p * kBlock, a.total - 1);
        const int ow = i % a.Wo, t = i / a.Wo;
        const int oh = t % a.Ho, plane = t / a.Ho;
        src[p] = a.x + (size_t)plane * a.H * a.W;
        const float* wt = a.w + (plane % a.C) * K * K;
        r0[p] = oh * S - K / 2, c0[p] = ow * S - K / 2;
#pragma unroll
        for (int q = 0; q < K * K; ++q) w[p][q] = wt[q];       // filter taps: not produced by any task
    }
    wait();
    if (!active) return;
#pragma unroll
    for (int p = 0; p < P; ++p) {
#pragma unroll
        for (int dr = 0; dr < K; ++dr)
#pragma unroll
            for (int dc = 0; dc < K; ++dc)
                v[p][dr * K + dc] = ldg(a.x, src[p] + min(max(r0[p] + dr, 0), a.H - 1) * a.W + min(max(c0[p] + dc, 0), a.W - 1), FIN);
    }
    __builtin_amdgcn_sched_barrier(0);                       // all loads are issued before the first use
#pragma unroll
    for (int p = 0; p < P; ++p) {
        float acc = 0.f;
#pragma unroll
        for (int dr = 0; dr < K; ++dr)
#pragma unroll
            for (int dc = 0; dc < K; ++dc) {
                const int r = r0[p] + dr, cc = c0[p] + dc;
                const bool in = r >= 0 && r < a.H && cc >= 0 && cc < a.W;
                acc = fmaf(w[p][dr * K + dc], in ? v[p][dr * K + dc] : 0.f, acc);
            }
        if (base + p * kBlock < a.total) stg(a.y, a.y + base + p * kBlock, acc, fout);
    }
}

// ------------------------------------------------------------------------------------
// global_avgpool: one wavefront per (n, c) plane, reduction across 64 lanes
// ------------------------------------------------------------------------------------
// Sum over the 64 lanes of a wavefront with data-parallel-primitive moves (one vector instruction per step, no trip
// through the LDS crossbar as a shuffle takes): a scan inside each row of 16 lanes (shifts by 1, 2, 4, 8, zeros shifted
// in) leaves a row's sum in its lane 15; lane 15 of rows 0 and 2 is then added to rows 1 and 3, lane 31 to rows 2 and 3,
// and lane 63 holds the total, which every lane gets back. The order of the additions is fixed.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, true);
    return v + __builtin_bit_cast(float, moved);
}
__device__ __forceinline__ float wave_sum(float v) {
    v = dpp_add<0x111, 0xf>(v);                              // row_shr:1
    v = dpp_add<0x112, 0xf>(v);                              // row_shr:2
    v = dpp_add<0x114, 0xf>(v);                              // row_shr:4
    v = dpp_add<0x118, 0xf>(v);                              // row_shr:8
    v = dpp_add<0x142, 0xa>(v);                              // row_bcast:15 into rows 1 and 3
    v = dpp_add<0x143, 0xc>(v);                              // row_bcast:31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

template <bool FIN, class Wait>
__device__ __forceinline__ void global_avgpool_tile(const GapArgs& a, int tile, float*, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    wait();
    const int lane = tid & 63;
    const int plane = tile * (kBlock / 64) + (tid >> 6);
    if (!live || plane >= a.planes) return;
    const float* src = a.x + (size_t)plane * a.HW;
    float acc = 0.f;
    for (int p = lane; p < a.HW; p += 64) acc += ldg(a.x, src + p, FIN);
    acc = wave_sum(acc);
    if (lane == 0) stg(a.y, a.y + plane, acc / (float)a.HW, fout);
}

// ------------------------------------------------------------------------------------
// fc (small batch): one wavefront per output feature; y[n][o] = <W[o], x[n]> + b[o]
// ------------------------------------------------------------------------------------
template <bool FIN, class Wait>
__device__ __forceinline__ void fc_gemv_tile(const FcArgs& a, int tile, float*, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    wait();
    const int lane = tid & 63;
    const int o = tile * (kBlock / 64) + (tid >> 6);
    if (!live || o >= a.Cout) return;
    const float* wr = a.w + (size_t)o * a.Cin;
    for (int n = 0; n < a.N; ++n) {
        const float* xr = a.x + (size_t)n * a.Cin;
        float acc = 0.f;
        if ((a.Cin & 3) == 0) {
            for (int k = lane * 4; k < a.Cin; k += 256) {
                const float4 wv = *reinterpret_cast<const float4*>(wr + k);
                const float4 xv = ldg4(a.x, xr + k, FIN);
                acc = fmaf(wv.x, xv.x, acc), acc = fmaf(wv.y, xv.y, acc);
                acc = fmaf(wv.z, xv.z, acc), acc = fmaf(wv.w, xv.w, acc);
            }
        } else {
            for (int k = lane; k < a.Cin; k += 64) acc = fmaf(wr[k], ldg(a.x, xr + k, FIN), acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) stg(a.y, a.y + (size_t)n * a.Cout + o, acc + a.b[o], fout);
    }
}

// ------------------------------------------------------------------------------------
// conv1x1 (and large-batch fc) on the matrix cores: Y[Cout x cols] = W[Cout x Cin] * X[Cin x cols]
// with cols = N * HW. v_mfma_f32_16x16x4_f32: A fragment lane l -> A[l % 16][l / 16],
// B fragment lane l -> B[l / 16][l % 16], accumulator register r of lane l -> D[4 * (l / 16) + r][l % 16].
// A workgroup of four wavefronts (2 x 2) owns a TM x TN output tile; K is walked in
// slices of KC staged through LDS, A as [k][m] so both fragments read rows. The weights are
// repacked at bind time into that order, W^T[CinP][CoutP] (zero padded; CinP a multiple of
// KC, CoutP of TM), so a slice of them is read and stored along m without any mask. Rows of
// the LDS slices are 16 (mod 32) floats apart: the four 16-lane groups of a wavefront, which
// read four consecutive rows, then hit different banks.
// ------------------------------------------------------------------------------------
template <int TM, int TN, int KC, bool FIN, class Wait>
__device__ __forceinline__ void conv1x1_mfma_tile(const PwArgs& a, int tile, float* smem, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    wait();
    constexpr int WM = TM / 2, WN = TN / 2;           // per-wavefront sub-tile
    constexpr int FM = WM / 16, FN = WN / 16;         // 16 x 16 fragments per wavefront
    constexpr int LDA = TM + 16, LDB = TN + 16;
    static_assert(LDA % 32 == 16 && LDB % 32 == 16, "row pitch of the LDS slices");
    static_assert(KC * (LDA + LDB) <= kSmemFloats, "LDS budget");
    static_assert(kBlock % TM == 0 && kBlock % TN == 0 && KC % (kBlock / TM) == 0 && KC % (kBlock / TN) == 0, "fill pattern");
    float* As = smem;                                 // [KC][LDA]
    float* Bs = smem + KC * LDA;                      // [KC][LDB]

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int by = tile / a.tiles_n, bx = tile - by * a.tiles_n;
    const int m0 = by * TM, n0 = bx * TN;

    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // A slice: W^T[k0 + k][m0 + m] -> As[k][m]; B slice: X[k0 + k][n0 + n] -> Bs[k][n]; consecutive
    // threads walk m and the pixels. Loads of X are unconditional from clamped indices (independent,
    // all in flight), zeroed when they are stored. The loads of slice k0 + KC are issued before the
    // matrix instructions of slice k0 and stored after them, so their latency overlaps with the arithmetic.
    constexpr int RA = kBlock / TM;                           // k rows of A covered per pass
    constexpr int RK = kBlock / TN;                           // k rows of B covered per pass
    const int CoutP = (a.Cout + TM - 1) / TM * TM;
    const float* wcol = a.wp + m0 + tid % TM + (size_t)(tid / TM) * CoutP;
    const int fn = tid % TN, fcol = n0 + fn;
    const int fccol = min(fcol, a.cols - 1);
    const int fimg = fccol / a.HW, fpix = fccol - fimg * a.HW;
    const float* xc = a.x + (size_t)fimg * a.Cin * a.HW + fpix;
    float va[KC / RA], vb[KC / RK];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < KC / RA; ++p) va[p] = wcol[(size_t)(k0 + p * RA) * CoutP];
#pragma unroll
        for (int p = 0; p < KC / RK; ++p) vb[p] = ldg(a.x, xc + (size_t)min(k0 + tid / TN + p * RK, a.Cin - 1) * a.HW, FIN);
    };
    if (live) fetch(0);
    for (int k0 = 0; k0 < a.Cin; k0 += KC) {
        if (live) {
#pragma unroll
            for (int p = 0; p < KC / RA; ++p) As[(tid / TM + p * RA) * LDA + tid % TM] = va[p];
#pragma unroll
            for (int p = 0; p < KC / RK; ++p) {
                const int k = tid / TN + p * RK;
                Bs[k * LDB + fn] = (fcol < a.cols && k0 + k < a.Cin) ? vb[p] : 0.f;
            }
        }
        __syncthreads();
        if (live && k0 + KC < a.Cin) fetch(k0 + KC);
        if (live)
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
            if (col >= a.cols || !live) continue;
            const int img = col / a.HW, pix = col - img * a.HW;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = m0 + wm * WM + i * 16 + 4 * (lane >> 4) + r;
                if (m < a.Cout) {
                    const float b = a.bias ? a.bias[m] : 0.f;
                    store_with_epilogue(a.y, a.ep, ((size_t)img * a.Cout + m) * a.HW + pix, m, acc[i][j][r] + b, fout);
                }
            }
        }
}

// ------------------------------------------------------------------------------------
// conv3x3 with many output columns (large maps, batches): the LDS-staged scheme of the kernel
// above on the implicit GEMM Y[Cout x cols] = W'[Cout x K'] * P[K' x cols], with K ordered tap
// first: k' = tap * CinP + ci, CinP = Cin rounded up to a multiple of KC. A K slice then has
// ONE tap, so where the slice's patch rows lie relative to a column (and whether that is inside
// the image) is worked out once per slice and thread, and the rows differ by a channel stride.
// The weights are repacked at bind time into W'^T[k'][CoutP] (zero padded; CoutP a multiple of
// TM), so a slice of them is read and stored to LDS along m without any mask. Rows of the LDS
// slices are 16 (mod 32) floats apart: the four 16-lane groups of a wavefront, which read four
// consecutive rows, then hit different banks. Every patch element is read from global memory
// once per workgroup tile instead of once per 16 x 16 MFMA tile.
// ------------------------------------------------------------------------------------
template <int TM, int TN, int KC, bool FIN, class Wait>
__device__ __forceinline__ void conv3x3_lds_tile(const C3Args& a, int tile, float* smem, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    constexpr int WM = TM / 2, WN = TN / 2;           // per-wavefront sub-tile
    constexpr int FM = WM / 16, FN = WN / 16;         // 16 x 16 fragments per wavefront
    constexpr int LDA = TM + 16, LDB = TN + 16;
    static_assert(LDA % 32 == 16 && LDB % 32 == 16, "row pitch of the LDS slices");
    static_assert(KC * (LDA + LDB) <= kSmemFloats, "LDS budget");
    static_assert(kBlock % TM == 0 && kBlock % TN == 0 && KC % (kBlock / TM) == 0 && KC % (kBlock / TN) == 0, "fill pattern");
    float* As = smem;                                 // [KC][LDA]
    float* Bs = smem + KC * LDA;                      // [KC][LDB]

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int by = tile / a.tiles_n, bx = tile - by * a.tiles_n;
    const int m0 = by * TM, n0 = bx * TN;
    const int CinP = a.groups, CoutP = (a.Cout + TM - 1) / TM * TM;
    const int HWo = a.Ho * a.Wo, HW = a.H * a.W;
    // the column this thread fills in every B slice
    const int fill_col = n0 + tid % TN;
    const int ccol = min(fill_col, a.cols - 1);
    const int fimg = ccol / HWo, fpix = ccol - fimg * HWo;
    const int foy = fpix / a.Wo, fox = fpix - foy * a.Wo;
    const int iy0 = foy * a.stride - a.pad, ix0 = fox * a.stride - a.pad;
    const float* xin = a.x + (size_t)fimg * a.Cin * HW;
    // the weight column this thread fills in every A slice
    constexpr int RA = kBlock / TM, RB = kBlock / TN;            // k rows covered per pass
    const float* wcol = a.wp + m0 + tid % TM + (size_t)(tid / TM) * CoutP;

    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    wait();

    for (int tap = 0; tap < 9; ++tap) {
        const int dr = tap / 3, dc = tap - 3 * dr;
        const int iy = iy0 + dr, ix = ix0 + dc;
        const bool inside = fill_col < a.cols && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
        const float* xtap = xin + min(max(iy, 0), a.H - 1) * a.W + min(max(ix, 0), a.W - 1);
        for (int c0 = 0; c0 < CinP; c0 += KC) {
            if (live) {
                float v[KC / RA], pv[KC / RB];
                const float* wk = wcol + (size_t)(tap * CinP + c0) * CoutP;
#pragma unroll
                for (int p = 0; p < KC / RA; ++p) v[p] = wk[(size_t)p * RA * CoutP];
#pragma unroll
                for (int p = 0; p < KC / RB; ++p) pv[p] = ldg(a.x, xtap + (size_t)min(c0 + tid / TN + p * RB, a.Cin - 1) * HW, FIN);
                __builtin_amdgcn_sched_barrier(0);               // all loads of the slice are issued before the first use
#pragma unroll
                for (int p = 0; p < KC / RA; ++p) As[(tid / TM + p * RA) * LDA + tid % TM] = v[p];
#pragma unroll
                for (int p = 0; p < KC / RB; ++p) {
                    const int kk = tid / TN + p * RB;
                    Bs[kk * LDB + tid % TN] = (inside && c0 + kk < a.Cin) ? pv[p] : 0.f;
                }
            }
            __syncthreads();
            if (live)
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
    }

#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int col = n0 + wn * WN + j * 16 + (lane & 15);
            if (col >= a.cols || !live) continue;
            const int img = col / HWo, pix = col - img * HWo;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = m0 + wm * WM + i * 16 + 4 * (lane >> 4) + r;
                if (m < a.Cout) store_with_epilogue(a.y, a.ep, ((size_t)img * a.Cout + m) * HWo + pix, m, acc[i][j][r], fout);
            }
        }
}

// ------------------------------------------------------------------------------------
// conv3x3 for many output pixels (large maps, batches), patch-stationary: Y[Cout x pixels] = W[Cout x 9 Cin] * patches.
// A tile is TM = 32 FM output channels by a run of TN = 32 FN consecutive output pixels of one image (row-major, so a run
// may wrap over several rows). K is walked in blocks of 16 input channels, and within a block tap by tap:
//   * B operand. The input pixels the run needs - its rows plus the halo, (W + 2 pad) wide with the padding stored as
//     zeros - are kept in LDS for one block of 16 channels, pixel-major, 20 floats per pixel, the 16 channels of a
//     pixel in the order p = 4 (k % 4) + k / 4: v_mfma_f32_16x16x4_f32 step s takes k = 4 s + g from lane group g, so
//     one 128-bit LDS read gives a lane its operands of all four steps. A tap is an address shift
//     ((dr (W + 2 pad) + dc) pixels), so the nine taps of a block run off ONE patch without a barrier between them: 9 x
//     4 FM FN matrix instructions per wavefront per pair of barriers, and each input element is fetched once per
//     tile and block instead of once per tap.
//   * A operand. The weights were repacked at bind time into [tap * blocks + block][CoutP][16] with the same order of
//     the 16 k: the 16 rows x 64 bytes a wavefront needs for one fragment are 1 KiB in a row, and every lane loads its
//     four operands with one 128-bit load straight from memory (L2) into registers, three slices ahead. No LDS, no
//     barrier and no vector ALU work for A.
//   * Filling the patch: a thread owns up to 4 PM / 256 (pixel, group of 4 channels) items; their global offsets are
//     worked out once per tile (out-of-image and padding positions get an offset beyond the buffer's size, for which
//     a buffer load returns 0), so a fill is four 32-bit loads with a scalar channel offset and one 128-bit LDS write
//     per item. The loads of block b + 1 are issued in the middle of block b's taps.
// Four wavefronts as 2 x 2, each 16 FM x 16 FN. Needs Cin % 16 == 0 and a patch of at most PM pixels.
// ------------------------------------------------------------------------------------
template <int FM, int FN, int PM, bool FIN, class Wait>
__device__ __forceinline__ void conv3x3_patch_tile(const C3Args& a, int tile, float* smem, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();
    constexpr int WM = 16 * FM, WN = 16 * FN, TM = 2 * WM, TN = 2 * WN, LD = 20;
    constexpr int ITEMS = 4 * PM / kBlock;
    constexpr unsigned kOutside = 0x80000000u;          // beyond any tensor (num_records < 2^31): the load returns 0
    constexpr int kIn = FIN ? kPolicyDeviceScope : 0;
    static_assert(PM * LD <= (PM > 256 ? kSmemFloatsWide : kSmemFloats) && PM % 64 == 0, "LDS budget");
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 15, g = lane >> 4;
    const int by = tile % a.co_groups, bt = tile / a.co_groups;
    const int img = bt / a.tiles_xy, seg = bt - img * a.tiles_xy;
    const int m0 = by * TM;
    const int HWo = a.Ho * a.Wo, HW = a.H * a.W;
    const int p0 = seg * TN, npx = min(TN, HWo - p0);
    const int oy_a = p0 / a.Wo, oy_b = (p0 + npx - 1) / a.Wo;
    const int iy_a = oy_a * a.stride - a.pad, Wp = a.W + 2 * a.pad, P = ((oy_b - oy_a) * a.stride + 3) * Wp;
    const int blocks = a.groups / 16, n_slices = 9 * blocks, CoutP = a.co_groups * TM;
    const __amdgpu_buffer_rsrc_t xr =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.x), 0, (a.tiles_n / a.tiles_xy) * a.Cin * HW * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.wp), 0, n_slices * CoutP * 64, 0x00020000);

    // this thread's fill items: (pixel of the patch, channels j, j + 4, j + 8, j + 12 of the block)
    unsigned goff[ITEMS];
    int loff[ITEMS];
#pragma unroll
    for (int t = 0; t < ITEMS; ++t) {
        const int idx = tid + kBlock * t;
        const int j = idx / P, pixel = idx - j * P;
        const int pr = pixel / Wp, pc = pixel - pr * Wp;
        const int iy = iy_a + pr, ix = pc - a.pad;
        const bool item = live && idx < 4 * P;
        const bool inside = item && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
        goff[t] = inside ? (unsigned)(((img * a.Cin + j) * HW + iy * a.W + ix) * 4) : kOutside;
        loff[t] = item ? pixel * (LD / 4) + j : -1;     // in units of 4 floats
    }
    // where this lane's B fragments start in the patch (tap 0), and its A rows in a slice of the packed weights
    int lbase[FN];
#pragma unroll
    for (int jn = 0; jn < FN; ++jn) {
        const int px = p0 + min(wn * WN + jn * 16 + r, npx - 1);
        const int oy = px / a.Wo, ox = px - oy * a.Wo;
        lbase[jn] = ((oy - oy_a) * a.stride * Wp + ox * a.stride) * LD + 4 * g;
    }
    const unsigned va_off = (unsigned)(((wm * WM + r) * 16 + 4 * g) * 4);

    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int jn = 0; jn < FN; ++jn) acc[i][jn] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 pv[ITEMS];
    // Loads are issued unconditionally and in a fixed order (idle items read "outside"): the compiler then counts
    // exactly how many younger loads may stay in flight at each wait.
    auto fill_load = [&](int block) {
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) {
            u32x4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = __builtin_amdgcn_raw_buffer_load_b32(xr, goff[t], (unsigned)((block * 16 + 4 * q) * HW * 4), kIn);
            pv[t] = v;
        }
    };
    auto fill_store = [&]() {
#pragma unroll
        for (int t = 0; t < ITEMS; ++t)
            if (loff[t] >= 0) reinterpret_cast<u32x4*>(smem)[loff[t]] = pv[t];
    };
    u32x4 af[3][FM];
    auto a_load = [&](int slice, int stage) {
        const int block = slice / 9, tap = slice - 9 * block;
        const unsigned so = (unsigned)(((tap * blocks + block) * CoutP + m0) * 64);
#pragma unroll
        for (int i = 0; i < FM; ++i) af[stage][i] = __builtin_amdgcn_raw_buffer_load_b128(wr, va_off + i * 1024, so, 0);
    };

    wait();
    if (live) {
        fill_load(0);
#pragma unroll
        for (int d = 0; d < 3; ++d) a_load(d, d);
        fill_store();
    }
    __syncthreads();
    for (int block = 0; block < blocks; ++block) {
        if (live) {
            f32x4 bf[2][FN];
#pragma unroll
            for (int jn = 0; jn < FN; ++jn) bf[0][jn] = *reinterpret_cast<const f32x4*>(smem + lbase[jn]);
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) {
                const int slice = block * 9 + tap, stage = tap % 3;
                if (tap < 8) {                          // next tap's B fragments, before this tap's matrix instructions
                    const int shift = (((tap + 1) / 3) * Wp + (tap + 1) % 3) * LD;
#pragma unroll
                    for (int jn = 0; jn < FN; ++jn) bf[(tap + 1) & 1][jn] = *reinterpret_cast<const f32x4*>(smem + lbase[jn] + shift);
                }
                if (tap == 3) {
                    fill_load(min(block + 1, blocks - 1));
                    __builtin_amdgcn_sched_barrier(0);  // keep the loads here: the compiler would sink them to their use
                }
                f32x4 afr[FM];
#pragma unroll
                for (int i = 0; i < FM; ++i) afr[i] = __builtin_bit_cast(f32x4, af[stage][i]);
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int jn = 0; jn < FN; ++jn)
                            acc[i][jn] = __builtin_amdgcn_mfma_f32_16x16x4f32(afr[i][s4], bf[tap & 1][jn][s4], acc[i][jn], 0, 0, 0);
                a_load(min(slice + 3, n_slices - 1), stage);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();                                // every wavefront is done with this block's patch
        if (live && block + 1 < blocks) fill_store();
        __syncthreads();
    }
    if (!live) return;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int jn = 0; jn < FN; ++jn) {
            const int cl = wn * WN + jn * 16 + r;
            if (cl >= npx) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int m = m0 + wm * WM + i * 16 + 4 * g + q;
                if (m < a.Cout) store_with_epilogue(a.y, a.ep, ((size_t)img * a.Cout + m) * HWo + p0 + cl, m, acc[i][jn][q], fout);
            }
        }
}

// W[Cout][Cin][3][3] -> [tap * (CinP / 16) + block][CoutP][16], the 16 channels of a block in the order
// p = 4 (k % 4) + k / 4 (position p holds k = 4 (p % 4) + p / 4); zero where m >= Cout or the channel >= Cin
__global__ __launch_bounds__(kBlock) void pack_c3_patch_weights_kernel(const float* w, float* wq, int Cout, int Cin, int CinP, int CoutP, long total) {
    const long idx = (long)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= total) return;
    const int p = (int)(idx & 15);
    const long row = idx >> 4;
    const int m = (int)(row % CoutP), slice = (int)(row / CoutP);
    const int kp = slice * 16 + 4 * (p & 3) + (p >> 2);
    const int tap = kp / CinP, ci = kp - tap * CinP;
    wq[idx] = (m < Cout && ci < Cin) ? w[((size_t)m * Cin + ci) * 9 + tap] : 0.f;
}

// ------------------------------------------------------------------------------------
// conv1x1 / fc for many output pixels on the plan of the patch-stationary conv3x3: Y[Cout x cols] = W[Cout x Cin] X[Cin x cols],
// tile = 32 FM output channels x 64 consecutive columns (a run may cross from one image into the next). KB blocks of 16
// input channels of the tile's columns sit in LDS, pixel-major (16 KB + 4 floats per column, the 16 channels of a block in
// the order the matrix instruction consumes them, so a lane's operands of four steps are one 128-bit read); the weights
// ([Cin / 16][CoutP][16], same channel order) go from memory straight into operands, one chunk ahead. Per pair of barriers
// a wavefront issues 8 KB FM matrix instructions. A thread fills one column's four-channel group per block: its global
// offset is worked out once per tile (columns beyond the end: an offset for which the buffer load returns 0).
// Four wavefronts as 2 x 2, each 16 FM x 32. Needs Cin % 16 == 0.
// ------------------------------------------------------------------------------------
template <int FM, int KB, bool FIN, class Wait>
__device__ __forceinline__ void conv1x1_patch_tile(const PwArgs& a, int tile, float* smem, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();
    constexpr int FN = 2, WM = 16 * FM, WN = 16 * FN, TM = 2 * WM, TN = 2 * WN, LD = 16 * KB + 4;
    constexpr unsigned kOutside = 0x80000000u;          // beyond any tensor (num_records < 2^31): the load returns 0
    constexpr int kIn = FIN ? kPolicyDeviceScope : 0;
    static_assert(TN * LD <= kSmemFloats && TN * 4 == kBlock, "LDS budget; one fill item per thread");
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, r = lane & 15, g = lane >> 4;
    const int by = tile % a.mtiles, bx = tile / a.mtiles;
    const int m0 = by * TM, n0 = bx * TN;
    const int blocks = a.ksteps / 16, chunks = (blocks + KB - 1) / KB, CoutP = a.mtiles * TM;
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.x), 0, a.cols * a.Cin * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.wp), 0, blocks * CoutP * 64, 0x00020000);
    // this thread's fill item: column c of the tile, channels j, j + 4, j + 8, j + 12 of every block
    unsigned goff;
    {
        const int c = tid % TN, j = tid / TN;
        const int col = n0 + c;
        const int img = col / a.HW, pix = col - img * a.HW;
        goff = (live && col < a.cols) ? (unsigned)(((img * a.Cin + j) * a.HW + pix) * 4) : kOutside;
    }
    const int loff = (tid % TN) * (LD / 4) + tid / TN;   // in units of 4 floats
    int lbase[FN];
#pragma unroll
    for (int jn = 0; jn < FN; ++jn) lbase[jn] = (wn * WN + jn * 16 + r) * LD + 4 * g;
    const unsigned va_off = (unsigned)(((wm * WM + r) * 16 + 4 * g) * 4);

    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int jn = 0; jn < FN; ++jn) acc[i][jn] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 pv[KB];
    // loads are issued unconditionally and in a fixed order (blocks beyond Cin read "outside"): the compiler then counts
    // exactly how many younger loads may stay in flight at each wait
    auto fill_load = [&](int chunk) {
#pragma unroll
        for (int b = 0; b < KB; ++b) {
            const int block = chunk * KB + b;
            const unsigned off = block < blocks ? goff : kOutside;
            u32x4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = __builtin_amdgcn_raw_buffer_load_b32(xr, off, (unsigned)((block * 16 + 4 * q) * a.HW * 4), kIn);
            pv[b] = v;
        }
    };
    auto fill_store = [&]() {
#pragma unroll
        for (int b = 0; b < KB; ++b) reinterpret_cast<u32x4*>(smem)[loff + 4 * b] = pv[b];
    };
    u32x4 af[KB][FM];
    auto a_load = [&](int slice, int stage) {           // a slice beyond Cin re-reads the last one: its activations are zeros
        const unsigned so = (unsigned)((min(slice, blocks - 1) * CoutP + m0) * 64);
#pragma unroll
        for (int i = 0; i < FM; ++i) af[stage][i] = __builtin_amdgcn_raw_buffer_load_b128(wr, va_off + i * 1024, so, 0);
    };

    wait();
    if (live) {
        fill_load(0);
#pragma unroll
        for (int b = 0; b < KB; ++b) a_load(b, b);
        fill_store();
    }
    __syncthreads();
    for (int chunk = 0; chunk < chunks; ++chunk) {
        if (live) {
            f32x4 bf[2][FN];
#pragma unroll
            for (int jn = 0; jn < FN; ++jn) bf[0][jn] = *reinterpret_cast<const f32x4*>(smem + lbase[jn]);
#pragma unroll
            for (int b = 0; b < KB; ++b) {
                if (b + 1 < KB) {
#pragma unroll
                    for (int jn = 0; jn < FN; ++jn) bf[(b + 1) & 1][jn] = *reinterpret_cast<const f32x4*>(smem + lbase[jn] + 16 * (b + 1));
                }
                if (b == 0) {
                    fill_load(min(chunk + 1, chunks - 1));
                    __builtin_amdgcn_sched_barrier(0);  // keep the loads here: the compiler would sink them to their use
                }
                f32x4 afr[FM];
#pragma unroll
                for (int i = 0; i < FM; ++i) afr[i] = __builtin_bit_cast(f32x4, af[b][i]);
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int jn = 0; jn < FN; ++jn)
                            acc[i][jn] = __builtin_amdgcn_mfma_f32_16x16x4f32(afr[i][s4], bf[b & 1][jn][s4], acc[i][jn], 0, 0, 0);
                a_load((chunk + 1) * KB + b, b);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();                                // every wavefront is done with this chunk
        if (live && chunk + 1 < chunks) fill_store();
        __syncthreads();
    }
    if (!live) return;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int jn = 0; jn < FN; ++jn) {
            const int col = n0 + wn * WN + jn * 16 + r;
            if (col >= a.cols) continue;
            const int img = col / a.HW, pix = col - img * a.HW;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int m = m0 + wm * WM + i * 16 + 4 * g + q;
                if (m < a.Cout)
                    store_with_epilogue(a.y, a.ep, ((size_t)img * a.Cout + m) * a.HW + pix, m, acc[i][jn][q] + (a.bias ? a.bias[m] : 0.f), fout);
            }
        }
}

// W[Cout][Cin] -> [Cin / 16][CoutP][16], the 16 channels of a block in the order p = 4 (k % 4) + k / 4; zero where m >= Cout
__global__ __launch_bounds__(kBlock) void pack_pw_patch_weights_kernel(const float* w, float* wq, int Cout, int Cin, int CoutP, long total) {
    const long idx = (long)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= total) return;
    const int p = (int)(idx & 15);
    const long row = idx >> 4;
    const int m = (int)(row % CoutP), block = (int)(row / CoutP);
    const int k = block * 16 + 4 * (p & 3) + (p >> 2);
    wq[idx] = (m < Cout && k < Cin) ? w[(size_t)m * Cin + k] : 0.f;
}

// W[Cout][Cin] -> W^T[CinP][CoutP], zero where k >= Cin or m >= Cout
__global__ __launch_bounds__(kBlock) void pack_pw_lds_weights_kernel(const float* w, float* wp, int Cout, int Cin, int CoutP, long total) {
    const long idx = (long)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= total) return;
    const int m = (int)(idx % CoutP), k = (int)(idx / CoutP);
    wp[idx] = (m < Cout && k < Cin) ? w[(size_t)m * Cin + k] : 0.f;
}

// W[Cout][Cin][3][3] -> W'^T[tap * CinP + ci][CoutP], zero where ci >= Cin or m >= Cout
__global__ __launch_bounds__(kBlock) void pack_c3_lds_weights_kernel(const float* w, float* wp, int Cout, int Cin, int CinP, int CoutP, long total) {
    const long idx = (long)blockIdx.x * kBlock + threadIdx.x;
    if (idx >= total) return;
    const int m = (int)(idx % CoutP);
    const int k = (int)(idx / CoutP);
    const int tap = k / CinP, ci = k - tap * CinP;
    wp[idx] = (m < Cout && ci < Cin) ? w[((size_t)m * Cin + ci) * 9 + tap] : 0.f;
}

// ------------------------------------------------------------------------------------
// conv1x1 for small problems (the batch-1 case): latency, not throughput, decides.
// A workgroup owns a 32 x 32 output tile as 2 x 2 MFMA tiles; its four wavefronts split K
// four ways, each accumulates all four MFMA tiles over its quarter of K with operands
// loaded straight from global memory into registers - no LDS staging and no barrier in
// the K loop, up to 64 loads in flight per lane - and the four partial results are summed
// through LDS in a fixed order (wavefront 0 + 1 + 2 + 3), so the result does not depend
// on timing. The weights are read from a copy repacked once, ahead of time, into the order
// the A operand wants: block (row tile rt, k step ks) holds W[16 rt + l % 16][4 ks + l / 16]
// for lane l = 0..63, zero outside the matrix, so one A load is one contiguous 256 bytes.
// The copy is zero-padded along K to a multiple of 4 x chunk steps: every wavefront runs
// whole chunks and the K loop needs no tail handling (a lone wavefront per SIMD issues one
// instruction every few cycles, so instruction count is what these kernels pay for).
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void pack_pw_weights_kernel(const float* w, float* wp, int Cout, int Cin,
                                                                  int ksteps, int total) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int l = i & 63, blk = i >> 6;
    const int ks = blk % ksteps, rt = blk / ksteps;
    const int m = rt * 16 + (l & 15), k = ks * 4 + (l >> 4);
    wp[i] = (m < Cout && k < Cin) ? w[(size_t)m * Cin + k] : 0.f;
}

template <int CH, bool FIN, class Wait>          // CH k steps per chunk: 4 * CH loads in flight per lane
__device__ __forceinline__ void conv1x1_direct_tile(const PwArgs& a, int tile, float* smem, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    wait();
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int by = tile / a.tiles_n, bx = tile - by * a.tiles_n;
    const int m0 = by * 32, n0 = bx * 32;
    const int S = a.ksteps;                                  // padded: every wavefront owns S / 4 steps, a multiple of CH
    const int steps = S >> 2;
    const unsigned k_last = (unsigned)(a.Cin - 1) * (unsigned)a.HW;   // offset of the last real input row
    const unsigned k_step = 4u * (unsigned)a.HW;

    const float* ap[2];
    const float* xb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int rt = min(by * 2 + i, a.mtiles - 1);       // a row tile past the matrix repeats the last one; never stored
        ap[i] = a.wp + ((size_t)rt * S + (size_t)wave * steps) * 64 + lane;
        const int col = min(n0 + i * 16 + (lane & 15), a.cols - 1);
        const int img = col / a.HW, pix = col - img * a.HW;
        xb[i] = a.x + (size_t)img * a.Cin * a.HW + pix;
    }
    // offset of this lane's input row at the wavefront's first step; rows past Cin (zero
    // weights there) are clamped onto the last real row so that every load stays in bounds
    unsigned koff = (unsigned)(4 * wave * steps + (lane >> 4)) * (unsigned)a.HW;
    f32x4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int s0 = 0; s0 < (live ? steps : 0); s0 += CH) {
        float av[2][CH], bv[2][CH];
#pragma unroll
        for (int q = 0; q < CH; ++q) {
            const unsigned off = min(koff + (unsigned)q * k_step, k_last);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                av[i][q] = ap[i][q * 64];
                bv[i][q] = ldg(a.x, xb[i] + off, FIN);
            }
        }
        __builtin_amdgcn_sched_barrier(0);                   // every load of the chunk is issued before the first use
#pragma unroll
        for (int q = 0; q < CH; ++q)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i][q], bv[j][q], acc[i][j], 0, 0, 0);
        ap[0] += CH * 64, ap[1] += CH * 64;
        koff += CH * k_step;
    }
    // partial sums -> LDS as red[wave][tile][reg][lane]; wavefront w then finishes MFMA tile w
    static_assert(4 * 4 * 4 * 64 <= kSmemFloats, "LDS budget");
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) smem[((wave * 4 + i * 2 + j) * 4 + r) * 64 + lane] = acc[i][j][r];
    __syncthreads();
    {
        const int ti = wave >> 1, tj = wave & 1;
        const int col = n0 + tj * 16 + (lane & 15);
        const int ccol = min(col, a.cols - 1);
        const int img = ccol / a.HW, pix = ccol - img * a.HW;
        float* yb = a.y + (size_t)img * a.Cout * a.HW + pix;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float sum = smem[((0 * 4 + wave) * 4 + r) * 64 + lane];
#pragma unroll
            for (int w2 = 1; w2 < 4; ++w2) sum += smem[((w2 * 4 + wave) * 4 + r) * 64 + lane];
            const int m = m0 + ti * 16 + 4 * (lane >> 4) + r;
            if (m < a.Cout && col < a.cols && live) {
                const float b = a.bias ? a.bias[m] : 0.f;
                store_with_epilogue(a.y, a.ep, (size_t)(yb - a.y) + (size_t)m * a.HW, m, sum + b, fout);
            }
        }
    }
    __syncthreads();                                         // LDS is reused by the next tile
}

// ------------------------------------------------------------------------------------
// conv1x1 for the smallest problems (one image, a few thousand pixels at most), where the
// time goes into issuing loads and into waiting, not into arithmetic. Differences from the
// 32 x 32 kernel above:
//   * the output tile is 16 channels wide only, so a problem spreads over as many compute
//     units as possible (an fp32 MFMA occupies its SIMD for 32 cycles: few tiles means
//     few SIMDs working);
//   * the packed weights hold 4 k-steps per lane (block (row tile, group g), lane l, word q
//     = W[16 rt + l % 16][16 g + 4 q + l / 16]): one 128-bit load feeds 4 MFMAs;
//   * VEC (pixels per plane a multiple of 4): activations are read 128 bits at a time. Lane l
//     loads X[k][n0 + 4 (l % 16) .. + 3]; word j of that load is the B operand of MFMA tile j,
//     whose columns are n0 + 4 i + j, i = 0..15 - four interleaved 16-column tiles, 64 columns
//     per workgroup, and the four results of a lane are again 4 consecutive pixels: one
//     128-bit store;
//   * otherwise the tile is 16 x 16 and activations are read word by word.
// K is split over the four wavefronts in groups of 4 k-steps, G groups in flight at a time;
// partial sums are added through LDS in a fixed order.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void pack_pw_weights_k4_kernel(const float* w, float* wp, int Cout, int Cin,
                                                                     int groups, int total) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int q = i & 3, l = (i >> 2) & 63, blk = i >> 8;
    const int gi = blk % groups, rt = blk / groups;
    const int m = rt * 16 + (l & 15), k = 16 * gi + 4 * q + (l >> 4);
    wp[i] = (m < Cout && k < Cin) ? w[(size_t)m * Cin + k] : 0.f;
}

template <int G, bool VEC, bool EA, bool FIN, class Wait>
__device__ __forceinline__ void conv1x1_k4_tile(const typename std::conditional<EA, PwAddArgs, PwArgs>::type& a, int tile, float* smem,
                                                int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    constexpr int NJ = VEC ? 4 : 1;                          // MFMA tiles per wavefront
    constexpr int TN = VEC ? 64 : 16;                        // columns per workgroup tile
    static_assert(4 * NJ * 4 * 64 <= kSmemFloats, "LDS budget");
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int by = tile / a.tiles_n, bx = tile - by * a.tiles_n;
    const int colv = bx * TN + (VEC ? 4 : 1) * (lane & 15);  // first column this lane owns
    // addresses first (nothing is read yet), then the wait for the producers
    const int groups = a.ksteps;                             // groups of 4 k-steps in the packed copy, a multiple of 4 G
    const int gw = groups >> 2;                              // groups per wavefront
    const f32x4* ap = reinterpret_cast<const f32x4*>(a.wp) + ((size_t)by * groups + (size_t)wave * gw) * 64 + lane;
    const int col = min(colv, a.cols - (VEC ? 4 : 1));       // columns past the end repeat the last ones; never stored
    const int img = col / a.HW, pix = col - img * a.HW;
    const float* xb = a.x + (size_t)img * a.Cin * a.HW + pix;
    const unsigned k_last = (unsigned)(a.Cin - 1) * (unsigned)a.HW;       // rows past Cin (zero weights) repeat the last row
    const unsigned k_step = 4u * (unsigned)a.HW;
    unsigned koff = (unsigned)(16 * wave * gw + (lane >> 4)) * (unsigned)a.HW;
    // wavefront w finishes accumulator register w of every MFMA tile: output row 4 (lane / 16) + w
    const int m = by * 16 + 4 * (lane >> 4) + wave;
    float es = 1.f, et = 0.f;
    if (a.ep.y != nullptr && a.ep.scale != nullptr) es = a.ep.scale[min(m, a.Cout - 1)], et = a.ep.shift[min(m, a.Cout - 1)];
    wait();
    if (live) {
        f32x4 acc[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int g0 = 0; g0 < gw; g0 += G) {
            f32x4 av[G];
            float bv[G][4][NJ];
#pragma unroll
            for (int gi = 0; gi < G; ++gi) {
                av[gi] = ap[gi * 64];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const unsigned off = min(koff + (unsigned)(4 * gi + q) * k_step, k_last);
                    if (VEC) {
                        const float4 v = ldg4(a.x, xb + off, FIN);
                        __builtin_memcpy(bv[gi][q], &v, sizeof v);
                    } else {
                        bv[gi][q][0] = ldg(a.x, xb + off, FIN);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);               // every load of the chunk is issued before the first use
#pragma unroll
            for (int gi = 0; gi < G; ++gi)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[gi][q], bv[gi][q][j], acc[j], 0, 0, 0);
            ap += G * 64;
            koff += 4u * G * k_step;
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) smem[((wave * NJ + j) * 4 + r) * 64 + lane] = acc[j][r];
    }
    __syncthreads();
    bool valid = false;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    size_t at = 0;
    if (live) {
        float out[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            float sum = smem[((0 * NJ + j) * 4 + wave) * 64 + lane];
#pragma unroll
            for (int w2 = 1; w2 < 4; ++w2) sum += smem[((w2 * NJ + j) * 4 + wave) * 64 + lane];
            out[j] = sum;
        }
        valid = m < a.Cout && colv < a.cols;                 // VEC: cols is a multiple of 4, a lane's 4 columns are all in or all out
        if (valid) {
            const float b = a.bias ? a.bias[m] : 0.f;
            const int img = colv / a.HW, pix = colv - img * a.HW;
            at = ((size_t)img * a.Cout + m) * a.HW + pix;
            v = make_float4(out[0] + b, out[NJ > 1 ? 1 : 0] + b, out[NJ > 2 ? 2 : 0] + b, out[NJ > 3 ? 3 : 0] + b);
            if (VEC) stg4(a.y, a.y + at, v, fout);
            else stg(a.y, a.y + at, v.x, fout);
            if (a.ep.y != nullptr) {
                v.x = fmaf(v.x, es, et), v.y = fmaf(v.y, es, et), v.z = fmaf(v.z, es, et), v.w = fmaf(v.w, es, et);
                if (a.ep.relu) v.x = fmaxf(v.x, 0.f), v.y = fmaxf(v.y, 0.f), v.z = fmaxf(v.z, 0.f), v.w = fmaxf(v.w, 0.f);
                if (VEC) stg4(a.ep.y, a.ep.y + at, v, fout);
                else stg(a.ep.y, a.ep.y + at, v.x, fout);
            }
        }
    }
    if constexpr (EA) {
        wait.late();
        if (valid) add_epilogue<VEC>(a.ea, v, at, fout);
    }
    __syncthreads();                                         // LDS is reused by the next tile
}

// ------------------------------------------------------------------------------------
// conv3x3 dense on the vector ALUs: one thread = one output pixel x 8 output channels.
// Input patches go through LDS (4 input channels per slice); the weights a wavefront
// needs are the same for all of its lanes, so they are read through uniform addresses.
// TP = 16: the workgroup owns a 16 x 16 pixel tile and one group of 8 output channels.
// TP = 8 : each wavefront owns the same 8 x 8 pixel tile and its own group of 8 channels.
// Tile index = (image * co_groups + channel group) * tiles_xy + pixel tile.
// ------------------------------------------------------------------------------------
template <int TP, int S, bool FIN, class Wait>
__device__ __forceinline__ void conv3x3_tile(const C3Args& a, int tile, float* smem, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    wait();
    constexpr int CIC = S == 2 && TP == 16 ? 2 : 4;    // input channels per LDS slice
    constexpr int IW = (TP - 1) * S + 3;               // input patch edge
    constexpr int LDP = IW + 1;
    constexpr int GROUPS = TP == 16 ? 1 : 4;           // channel groups per workgroup
    constexpr int CO = 8;
    constexpr int WROW = 12;                           // a (channel, input channel) pair's nine taps, padded to three 128-bit reads
    constexpr int NW = GROUPS * CO * CIC;              // such pairs per slice
    static_assert(CIC * IW * LDP + NW * WROW <= kSmemFloats && (CIC * IW * LDP) % 4 == 0, "LDS budget; the weights start 16-byte aligned");
    float* patch = smem;                               // [CIC][IW][LDP]
    float* wsm = smem + CIC * IW * LDP;                // [GROUPS CO][CIC][WROW]: the slice's weights of every output channel of the workgroup

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
    // The weights go through LDS with the patch (one batch of loads, one barrier): read through uniform addresses
    // straight from memory they arrived a few at a time, each batch a trip to L2 that the wavefront waited for, and
    // that, not arithmetic or bandwidth, was the tile's 8 us on a stem. Out-of-range channels repeat the last one and are
    // masked at the store.
    const int cbase = cog * GROUPS * CO;               // first output channel of the workgroup
    const int wgroup = TP == 16 ? 0 : wave;

    for (int c0 = 0; c0 < a.Cin; c0 += CIC) {
        if (live) {
            constexpr int NL = (CIC * IW * IW + kBlock - 1) / kBlock;   // loads per thread, all in flight
            float pv[NL];
#pragma unroll
            for (int q = 0; q < NL; ++q) {
                const int e = min(tid + q * kBlock, CIC * IW * IW - 1);
                const int cx = e % IW, t = e / IW;
                const int cy = t % IW, ci = t / IW;
                const int gy = iy0 + cy, gx = ix0 + cx, gc = c0 + ci;
                const bool in = gc < a.Cin && gy >= 0 && gy < a.H && gx >= 0 && gx < a.W;
                const float v = ldg(a.x, xin + ((size_t)min(gc, a.Cin - 1) * a.H + min(max(gy, 0), a.H - 1)) * a.W + min(max(gx, 0), a.W - 1), FIN);
                pv[q] = in ? v : 0.f;
            }
            constexpr int NWL = (NW * 9 + kBlock - 1) / kBlock;         // weight loads per thread
            float wv[NWL];
#pragma unroll
            for (int q = 0; q < NWL; ++q) {
                const int e = min(tid + q * kBlock, NW * 9 - 1);
                const int tap = e % 9, pair = e / 9, ci = pair % CIC, jj = pair / CIC;
                const float v = a.w[((size_t)min(cbase + jj, a.Cout - 1) * a.Cin + min(c0 + ci, a.Cin - 1)) * 9 + tap];
                wv[q] = c0 + ci < a.Cin ? v : 0.f;
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < NL; ++q) {
                const int e = tid + q * kBlock;
                if (e < CIC * IW * IW) {
                    const int cx = e % IW, t = e / IW;
                    const int cy = t % IW, ci = t / IW;
                    patch[(ci * IW + cy) * LDP + cx] = pv[q];
                }
            }
#pragma unroll
            for (int q = 0; q < NWL; ++q) {
                const int e = tid + q * kBlock;
                if (e < NW * 9) wsm[(e / 9) * WROW + e % 9] = wv[q];
            }
        }
        __syncthreads();
        const int nci = live ? min(CIC, a.Cin - c0) : 0;
        for (int ci = 0; ci < nci; ++ci) {
            float in[9];
#pragma unroll
            for (int dr = 0; dr < 3; ++dr)
#pragma unroll
                for (int dc = 0; dc < 3; ++dc) in[dr * 3 + dc] = patch[(ci * IW + ty * S + dr) * LDP + tx * S + dc];
#pragma unroll
            for (int j = 0; j < CO; ++j) {
                const float4* wp = reinterpret_cast<const float4*>(wsm + ((wgroup * CO + j) * CIC + ci) * WROW);   // the same address in every lane: a broadcast
                const float4 w0 = wp[0], w1 = wp[1], w2 = wp[2];
                const float wq[9] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w, w2.x};
#pragma unroll
                for (int q = 0; q < 9; ++q) acc[j] = fmaf(wq[q], in[q], acc[j]);
            }
        }
        __syncthreads();
    }
    if (oy < a.Ho && ox < a.Wo && live) {
#pragma unroll
        for (int j = 0; j < CO; ++j)
            if (co0 + j < a.Cout)
                store_with_epilogue(a.y, a.ep, (((size_t)img * a.Cout + co0 + j) * a.Ho + oy) * a.Wo + ox, co0 + j, acc[j], fout);
    }
}

// ------------------------------------------------------------------------------------
// conv3x3 as an implicit GEMM on the matrix cores: Y[Cout x cols] = W[Cout x 9 Cin] * P[9 Cin x cols]
// with cols = N * Ho * Wo and P[(ci, dr, dc)][(n, oy, ox)] = x[n][ci][oy S - pad + dr][ox S - pad + dc]
// (zero outside the image), gathered straight from global memory: the weight tensor
// [Cout][Cin][3][3] already is that W, row-major, so it is repacked exactly like a 1x1
// weight matrix with 9 Cin input channels. Same structure as the 16 x 16 conv1x1 above: K split
// over the four wavefronts in groups of 4 k-steps, G groups in flight, fixed-order reduction.
// A lane walks k in steps of 4, so (ci, tap) is updated incrementally: tap += 4, carry into ci.
// ------------------------------------------------------------------------------------
template <int G, bool EA, bool FIN, class Wait>
__device__ __forceinline__ void conv3x3_k4_tile(const typename std::conditional<EA, C3AddArgs, C3Args>::type& a, int tile, float* smem,
                                                int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();       // device-scope stores: some reader of the result sits on another XCD
    static_assert(4 * 4 * 64 <= kSmemFloats, "LDS budget");
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int by = tile / a.tiles_n, bx = tile - by * a.tiles_n;
    const int colv = bx * 16 + (lane & 15);
    const int HWo = a.Ho * a.Wo;
    // addresses first (nothing is read yet), then the wait for the producers
    const int groups = a.groups, gw = groups >> 2;
    const f32x4* ap = reinterpret_cast<const f32x4*>(a.wp) + ((size_t)by * groups + (size_t)wave * gw) * 64 + lane;
    const int col = min(colv, a.cols - 1);                   // columns past the end repeat the last one; never stored
    const int img = col / HWo, pix = col - img * HWo;
    const int oy = pix / a.Wo, ox = pix - oy * a.Wo;
    const int iy0 = oy * a.stride - a.pad, ix0 = ox * a.stride - a.pad;
    const int HW = a.H * a.W;
    const float* xb = a.x + (size_t)img * a.Cin * HW;
    const int k0 = 16 * wave * gw + (lane >> 4);             // this lane's first k; then + 4 per k-step
    int ci = k0 / 9, tap = k0 - 9 * ci;
    const int m = by * 16 + 4 * (lane >> 4) + wave;          // wavefront w finishes accumulator register w
    float es = 1.f, et = 0.f;
    if (a.ep.y != nullptr && a.ep.scale != nullptr) es = a.ep.scale[min(m, a.Cout - 1)], et = a.ep.shift[min(m, a.Cout - 1)];
    wait();
    if (live) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int g0 = 0; g0 < gw; g0 += G) {
            f32x4 av[G];
            float bv[G][4];
            unsigned inside = 0;
#pragma unroll
            for (int gi = 0; gi < G; ++gi) {
                av[gi] = ap[gi * 64];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int dr = (tap * 11) >> 5, dc = tap - 3 * dr;       // tap / 3, tap % 3 for tap < 9
                    const int iy = iy0 + dr, ix = ix0 + dc;
                    const bool in = ci < a.Cin && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
                    inside |= (in ? 1u : 0u) << (gi * 4 + q);
                    const int off = min(ci, a.Cin - 1) * HW + min(max(iy, 0), a.H - 1) * a.W + min(max(ix, 0), a.W - 1);
                    bv[gi][q] = ldg(a.x, xb + off, FIN);
                    tap += 4;
                    if (tap >= 9) tap -= 9, ++ci;
                }
            }
            __builtin_amdgcn_sched_barrier(0);               // every load of the chunk is issued before the first use
#pragma unroll
            for (int gi = 0; gi < G; ++gi)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[gi][q], ((inside >> (gi * 4 + q)) & 1u) ? bv[gi][q] : 0.f, acc, 0, 0, 0);
            ap += G * 64;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) smem[(wave * 4 + r) * 64 + lane] = acc[r];
    }
    __syncthreads();
    bool valid = false;
    float z = 0.f;
    size_t at = 0;
    if (live) {
        float sum = smem[(0 * 4 + wave) * 64 + lane];
#pragma unroll
        for (int w2 = 1; w2 < 4; ++w2) sum += smem[(w2 * 4 + wave) * 64 + lane];
        valid = m < a.Cout && colv < a.cols;
        if (valid) {
            const int img = colv / HWo, pix = colv - img * HWo;
            at = ((size_t)img * a.Cout + m) * HWo + pix;
            stg(a.y, a.y + at, sum, fout);
            z = sum;
            if (a.ep.y != nullptr) {
                z = fmaf(sum, es, et);
                if (a.ep.relu) z = fmaxf(z, 0.f);
                stg(a.ep.y, a.ep.y + at, z, fout);
            }
        }
    }
    if constexpr (EA) {
        wait.late();
        if (valid) add_epilogue<false>(a.ea, make_float4(z, 0.f, 0.f, 0.f), at, fout);
    }
    __syncthreads();                                         // LDS is reused by the next tile
}

// ------------------------------------------------------------------------------------
// pool3x3 for large tensors (batches): a thread computes 4 outputs of one output column, one below the other;
// neighbouring lanes have neighbouring columns, so every load and store of a wavefront is a contiguous run. The 3 + 3 STRIDE
// input rows x 3 columns the four windows cover are loaded once (4.5 loads per output at stride 1 instead of 9, each
// touching 2-3 cache lines per wavefront), reduced along the rows first and then down the column; row / column validity
// is worked out once per thread. Items = (plane, block of 4 output rows, output column) in that order.
// (Four neighbouring outputs of a ROW per thread was measured first and is slower than one output per thread: lanes
// 16 bytes apart make every load instruction touch eight cache lines.)
// ------------------------------------------------------------------------------------
template <int STRIDE, bool FIN, class Wait>
__device__ __forceinline__ void pool3x3_col_tile(const PoolArgs& a, int tile, float*, int tid, bool live, Wait& wait) {
    const bool fout = wait.far_out();
    constexpr int NR = 3 + 3 * STRIDE;                       // input rows under four windows one below the other
    const int blocks = (a.Ho + 3) >> 2;
    const int items = (a.total / (a.Ho * a.Wo)) * blocks * a.Wo;
    const int item = tile * kBlock + tid;
    const bool active = live && item < items;
    const int it = min(item, items - 1);
    const int ow = it % a.Wo, t1 = it / a.Wo;
    const int blk = t1 % blocks, plane = t1 / blocks;
    const int oh0 = 4 * blk, r0 = oh0 * STRIDE - a.pad, c0 = ow * STRIDE - a.pad;
    const float* src = a.x + (size_t)plane * a.H * a.W;
    wait();
    if (!active) return;
    const bool max_mode = a.mode == 0;
    const float neutral = max_mode ? -INFINITY : 0.f;
    float v[NR][3];
    bool row_in[NR], col_in[3];
#pragma unroll
    for (int dr = 0; dr < NR; ++dr) row_in[dr] = (unsigned)(r0 + dr) < (unsigned)a.H;
#pragma unroll
    for (int dc = 0; dc < 3; ++dc) col_in[dc] = (unsigned)(c0 + dc) < (unsigned)a.W;
    int cc[3];
#pragma unroll
    for (int dc = 0; dc < 3; ++dc) cc[dc] = min(max(c0 + dc, 0), a.W - 1);
#pragma unroll
    for (int dr = 0; dr < NR; ++dr) {
        const float* row = src + min(max(r0 + dr, 0), a.H - 1) * a.W;
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) v[dr][dc] = ldg(a.x, row + cc[dc], FIN);
    }
    __builtin_amdgcn_sched_barrier(0);                       // all loads are issued before the first use
    float rowv[NR];                                          // along the rows: columns outside the image do not take part
#pragma unroll
    for (int dr = 0; dr < NR; ++dr) {
        float acc = neutral;
#pragma unroll
        for (int dc = 0; dc < 3; ++dc) {
            const float x = col_in[dc] ? v[dr][dc] : neutral;
            acc = max_mode ? fmaxf(acc, x) : acc + x;
        }
        rowv[dr] = row_in[dr] ? acc : neutral;
    }
    const int cols = (int)col_in[0] + (int)col_in[1] + (int)col_in[2];
    float* out = a.y + ((size_t)plane * a.Ho + oh0) * a.Wo + ow;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (oh0 + j >= a.Ho) break;
        const int b = j * STRIDE;
        float acc = max_mode ? fmaxf(fmaxf(rowv[b], rowv[b + 1]), rowv[b + 2]) : (rowv[b] + rowv[b + 1]) + rowv[b + 2];
        if (!max_mode) acc = acc / (float)(cols * ((int)row_in[b] + (int)row_in[b + 1] + (int)row_in[b + 2]));
        stg(a.y, out + (size_t)j * a.Wo, acc, fout);
    }
}

// ------------------------------------------------------------------------------------
// dwconv for large tensors of small planes (batches of CIFAR-sized maps): a workgroup takes as many whole
// (image, channel) planes as fit 1024 input pixels, stages them in LDS with a border of zeros (one 128-bit load per
// thread; the taps then need no bounds and no index arithmetic beyond a row pitch) and every thread computes four
// outputs side by side from K rows of 3 S + K values, stored with one 128-bit store.
// ------------------------------------------------------------------------------------
template <int K, int S, bool FIN, class Wait>
__device__ __forceinline__ void dwconv_lds_impl(const DwArgs& a, int tile, float* smem, int tid, bool live, Wait& wait) {
    constexpr int p = K / 2, SPAN = 3 * S + K;
    const bool fout = wait.far_out();
    const int HW = a.H * a.W, HWo = a.Ho * a.Wo;
    const int PW = a.W + 2 * p, PHW = (a.H + 2 * p) * PW;
    const int G = a.planes_per_tile;
    const int p0 = tile * G, np = live ? min(G, a.total / HWo - p0) : 0;
    const int xq = 4 * tid, gi = xq / HW, xrem = xq - gi * HW, iy = xrem / a.W, ix = xrem - iy * a.W;
    const int oq = 4 * tid, go = oq / HWo, orem = oq - go * HWo, oy = orem / a.Wo, ox = orem - oy * a.Wo;
    const bool xin = gi < np, oin = go < np;
    float w[K * K];
    const float* wt = a.w + ((p0 + min(go, max(np - 1, 0))) % a.C) * (K * K);
#pragma unroll
    for (int q = 0; q < K * K; ++q) w[q] = wt[q];              // filter taps: not produced by any task
    wait();
    const float4 x4 = xin ? ldg4(a.x, a.x + (size_t)p0 * HW + xq, FIN) : make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();                                            // a previous tile of this workgroup has been read to the end
    for (int i = tid; i < G * PHW; i += kBlock) smem[i] = 0.f;
    __syncthreads();
    if (xin) {
        float* dst = smem + gi * PHW + (iy + p) * PW + ix + p;
        dst[0] = x4.x, dst[1] = x4.y, dst[2] = x4.z, dst[3] = x4.w;
    }
    __syncthreads();
    if (!oin) return;
    const float* src = smem + go * PHW + oy * S * PW + ox * S;  // tap (0, 0) of the first of the four outputs
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int da = 0; da < K; ++da) {
        float v[SPAN];
#pragma unroll
        for (int s = 0; s < SPAN; ++s) v[s] = src[da * PW + s];
#pragma unroll
        for (int db = 0; db < K; ++db)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = fmaf(w[da * K + db], v[j * S + db], acc[j]);   // taps in ascending order, as dwconv_tile
    }
    stg4(a.y, a.y + (size_t)p0 * HWo + oq, make_float4(acc[0], acc[1], acc[2], acc[3]), fout);
}
template <bool FIN, class Wait>
__device__ __forceinline__ void dwconv_lds_tile(const DwArgs& a, int tile, float* smem, int tid, bool live, Wait& wait) {
    if (a.K == 3 && a.S == 1) dwconv_lds_impl<3, 1, FIN>(a, tile, smem, tid, live, wait);
    else if (a.K == 3) dwconv_lds_impl<3, 2, FIN>(a, tile, smem, tid, live, wait);
    else if (a.S == 1) dwconv_lds_impl<5, 1, FIN>(a, tile, smem, tid, live, wait);
    else dwconv_lds_impl<5, 2, FIN>(a, tile, smem, tid, live, wait);
}

#include "ng_train_tiles.inc"

// ------------------------------------------------------------------------------------
// kernel table: id -> argument type, tile function, name
// ------------------------------------------------------------------------------------
// FIN: activations are read with device-scope loads (some operand was produced on another
// XCD) - a template argument, because loads sit in the inner loops. Whether the result is stored
// with device-scope stores (some reader sits on another XCD) is a run-time property of the
// `wait` object: a kernel has a handful of stores, and one variant less per kernel halves the code.
template <int KID> struct KernelOf;
#define NG_KERNEL(KID, ARGS, NAME, ...)                                                        \
    template <> struct KernelOf<KID> {                                                         \
        using Args = ARGS;                                                                     \
        static constexpr const char* name = NAME;                                              \
        template <bool FIN, class Wait>                                                        \
        static __device__ __forceinline__ void tile(const ARGS& a, int t, float* smem, int tid, bool live, Wait& wait) { \
            __VA_ARGS__, FIN > (a, t, smem, tid, live, wait);                                  \
        }                                                                                      \
    };
NG_KERNEL(KID_BN, BnArgs, "bn_act", bn_act_tile < PART_L256)
NG_KERNEL(KID_BN_V4, BnArgs, "bn_act_v4", bn_act_tile < PART_L1024)
NG_KERNEL(KID_BN_R64, BnArgs, "bn_act_r64", bn_act_tile < PART_R64)
NG_KERNEL(KID_BN_R16, BnArgs, "bn_act_r16", bn_act_tile < PART_R16)
NG_KERNEL(KID_ADD_R64, AddArgs, "add_n_r64", add_n_tile < PART_R64)
NG_KERNEL(KID_ADD_R16, AddArgs, "add_n_r16", add_n_tile < PART_R16)
NG_KERNEL(KID_ADD, AddArgs, "add_n", add_n_tile < PART_L256)
NG_KERNEL(KID_ADD_V4, AddArgs, "add_n_v4", add_n_tile < PART_L1024)
NG_KERNEL(KID_CONCAT, ConcatArgs, "concat", concat_tile < false)
NG_KERNEL(KID_CONCAT_V4, ConcatArgs, "concat_v4", concat_tile < true)
NG_KERNEL(KID_DW_K3S1, DwArgs, "dwconv_k3s1", dwconv_tile < 3, 1, 1)
NG_KERNEL(KID_DW_K3S2, DwArgs, "dwconv_k3s2", dwconv_tile < 3, 2, 1)
NG_KERNEL(KID_DW_K5S1, DwArgs, "dwconv_k5s1", dwconv_tile < 5, 1, 1)
NG_KERNEL(KID_DW_K5S2, DwArgs, "dwconv_k5s2", dwconv_tile < 5, 2, 1)
NG_KERNEL(KID_DW_K3S1_P4, DwArgs, "dwconv_k3s1_p4", dwconv_tile < 3, 1, 4)
NG_KERNEL(KID_POOL, PoolArgs, "pool3x3", pool3x3_tile < 1, false)
NG_KERNEL(KID_POOL_P4, PoolArgs, "pool3x3_p4", pool3x3_tile < 4, false)
NG_KERNEL(KID_POOL_ROW_S1, PoolArgs, "pool3x3_col4_s1", pool3x3_col_tile < 1)
NG_KERNEL(KID_POOL_ROW_S2, PoolArgs, "pool3x3_col4_s2", pool3x3_col_tile < 2)
NG_KERNEL(KID_POOL_A, PoolAddArgs, "pool3x3_add", pool3x3_tile < 1, true)
NG_KERNEL(KID_POOL_P4A, PoolAddArgs, "pool3x3_p4_add", pool3x3_tile < 4, true)
NG_KERNEL(KID_PW_D4, PwArgs, "conv1x1_mfma_d4", conv1x1_direct_tile < 4)
NG_KERNEL(KID_PW_D8, PwArgs, "conv1x1_mfma_d8", conv1x1_direct_tile < 8)
NG_KERNEL(KID_PW_D16, PwArgs, "conv1x1_mfma_d16", conv1x1_direct_tile < 16)
NG_KERNEL(KID_PW_64, PwArgs, "conv1x1_mfma_64x64", conv1x1_mfma_tile < 64, 64, 16)
NG_KERNEL(KID_PW_V1, PwArgs, "conv1x1_v1", conv1x1_k4_tile < 1, true, false)
NG_KERNEL(KID_PW_V2, PwArgs, "conv1x1_v2", conv1x1_k4_tile < 2, true, false)
NG_KERNEL(KID_PW_V3, PwArgs, "conv1x1_v3", conv1x1_k4_tile < 3, true, false)
NG_KERNEL(KID_PW_V4, PwArgs, "conv1x1_v4", conv1x1_k4_tile < 4, true, false)
NG_KERNEL(KID_PW_S1, PwArgs, "conv1x1_s1", conv1x1_k4_tile < 1, false, false)
NG_KERNEL(KID_PW_S2, PwArgs, "conv1x1_s2", conv1x1_k4_tile < 2, false, false)
NG_KERNEL(KID_PW_S3, PwArgs, "conv1x1_s3", conv1x1_k4_tile < 3, false, false)
NG_KERNEL(KID_PW_S4, PwArgs, "conv1x1_s4", conv1x1_k4_tile < 4, false, false)
NG_KERNEL(KID_C3_T16S1, C3Args, "conv3x3_t16s1", conv3x3_tile < 16, 1)
NG_KERNEL(KID_C3_T16S2, C3Args, "conv3x3_t16s2", conv3x3_tile < 16, 2)
NG_KERNEL(KID_C3_T8S1, C3Args, "conv3x3_t8s1", conv3x3_tile < 8, 1)
NG_KERNEL(KID_C3_T8S2, C3Args, "conv3x3_t8s2", conv3x3_tile < 8, 2)
NG_KERNEL(KID_C3_M1, C3Args, "conv3x3_mfma_1", conv3x3_k4_tile < 1, false)
NG_KERNEL(KID_C3_M2, C3Args, "conv3x3_mfma_2", conv3x3_k4_tile < 2, false)
NG_KERNEL(KID_C3_M3, C3Args, "conv3x3_mfma_3", conv3x3_k4_tile < 3, false)
NG_KERNEL(KID_C3_M4, C3Args, "conv3x3_mfma_4", conv3x3_k4_tile < 4, false)
NG_KERNEL(KID_PW_V1A, PwAddArgs, "conv1x1_v1_add", conv1x1_k4_tile < 1, true, true)
NG_KERNEL(KID_PW_V2A, PwAddArgs, "conv1x1_v2_add", conv1x1_k4_tile < 2, true, true)
NG_KERNEL(KID_PW_V3A, PwAddArgs, "conv1x1_v3_add", conv1x1_k4_tile < 3, true, true)
NG_KERNEL(KID_PW_V4A, PwAddArgs, "conv1x1_v4_add", conv1x1_k4_tile < 4, true, true)
NG_KERNEL(KID_PW_S1A, PwAddArgs, "conv1x1_s1_add", conv1x1_k4_tile < 1, false, true)
NG_KERNEL(KID_PW_S2A, PwAddArgs, "conv1x1_s2_add", conv1x1_k4_tile < 2, false, true)
NG_KERNEL(KID_PW_S3A, PwAddArgs, "conv1x1_s3_add", conv1x1_k4_tile < 3, false, true)
NG_KERNEL(KID_PW_S4A, PwAddArgs, "conv1x1_s4_add", conv1x1_k4_tile < 4, false, true)
NG_KERNEL(KID_C3_M1A, C3AddArgs, "conv3x3_mfma_1_add", conv3x3_k4_tile < 1, true)
NG_KERNEL(KID_C3_M2A, C3AddArgs, "conv3x3_mfma_2_add", conv3x3_k4_tile < 2, true)
NG_KERNEL(KID_C3_M3A, C3AddArgs, "conv3x3_mfma_3_add", conv3x3_k4_tile < 3, true)
NG_KERNEL(KID_C3_M4A, C3AddArgs, "conv3x3_mfma_4_add", conv3x3_k4_tile < 4, true)
NG_KERNEL(KID_C3_L32, C3Args, "conv3x3_lds_32x128", conv3x3_lds_tile < 32, 128, 16)
NG_KERNEL(KID_C3_L64, C3Args, "conv3x3_lds_64x64", conv3x3_lds_tile < 64, 64, 32)
NG_KERNEL(KID_PW_P32, PwArgs, "conv1x1_patch_32x64", conv1x1_patch_tile < 1, 4)
NG_KERNEL(KID_PW_P64, PwArgs, "conv1x1_patch_64x64", conv1x1_patch_tile < 2, 2)
NG_KERNEL(KID_C3_P64, C3Args, "conv3x3_patch_64x64", conv3x3_patch_tile < 2, 2, 256)
NG_KERNEL(KID_C3_P96, C3Args, "conv3x3_patch_96x64", conv3x3_patch_tile < 3, 2, 256)
NG_KERNEL(KID_C3_Q32, C3Args, "conv3x3_patch_32x128_wide", conv3x3_patch_tile < 1, 4, 640)
NG_KERNEL(KID_C3_Q64, C3Args, "conv3x3_patch_64x64_wide", conv3x3_patch_tile < 2, 2, 640)
NG_KERNEL(KID_C3_Q128, C3Args, "conv3x3_patch_64x128_wide", conv3x3_patch_tile < 2, 4, 640)
NG_KERNEL(KID_GEMM_PW_FWD, GemmArgs, "gemm_conv1x1_fwd", gemm_tile < GEMM_PW_FWD)
NG_KERNEL(KID_GEMM_PW_DGRAD, GemmArgs, "gemm_conv1x1_dgrad", gemm_tile < GEMM_PW_DGRAD)
NG_KERNEL(KID_GEMM_PW_WGRAD, GemmArgs, "gemm_conv1x1_wgrad", gemm_tile < GEMM_PW_WGRAD)
NG_KERNEL(KID_PW_WGRAD_PX, GemmArgs, "conv1x1_wgrad_px_16", pw_wgrad_px_tile < 1, false)
NG_KERNEL(KID_PW_WGRAD_PX2, GemmArgs, "conv1x1_wgrad_px_32", pw_wgrad_px_tile < 2, false)
NG_KERNEL(KID_C3_WGRAD_PX, GemmArgs, "conv3x3_wgrad_px_16", pw_wgrad_px_tile < 1, true)
NG_KERNEL(KID_C3_WGRAD_PX2, GemmArgs, "conv3x3_wgrad_px_32", pw_wgrad_px_tile < 2, true)
NG_KERNEL(KID_PW_PX_FWD, GemmArgs, "conv1x1_px_fwd", pw_px_tile < GEMM_PW_FWD)
NG_KERNEL(KID_PW_PX_DGRAD, GemmArgs, "conv1x1_px_dgrad", pw_px_tile < GEMM_PW_DGRAD)
NG_KERNEL(KID_GEMM_C3_FWD, GemmArgs, "gemm_conv3x3_fwd", gemm_tile < GEMM_C3_FWD)
NG_KERNEL(KID_GEMM_C3_DGRAD, GemmArgs, "gemm_conv3x3_dgrad", gemm_tile < GEMM_C3_DGRAD)
NG_KERNEL(KID_GEMM_C3_WGRAD, GemmArgs, "gemm_conv3x3_wgrad", gemm_tile < GEMM_C3_WGRAD)
NG_KERNEL(KID_BN_RAW, BnRawArgs, "bn_act_raw", bn_raw_tile < 0)
NG_KERNEL(KID_BN_DGRAD, BnRawArgs, "bn_act_dgrad", bn_raw_tile < 1)
NG_KERNEL(KID_BN_WGRAD, BnRawArgs, "bn_act_wgrad", bn_wgrad_tile < false)
NG_KERNEL(KID_BN_BACKWARD, BnRawArgs, "bn_act_backward", bn_wgrad_tile < true)
NG_KERNEL(KID_RELU_DGRAD, EltGradArgs, "relu_dgrad", elt_grad_tile < 0)
NG_KERNEL(KID_GAP_DGRAD, EltGradArgs, "global_avgpool_dgrad", elt_grad_tile < 1)
NG_KERNEL(KID_SLICE_PAD, EltGradArgs, "slice_pad", elt_grad_tile < 2)
#undef NG_KERNEL
// kernels without further template arguments
#define NG_KERNEL0(KID, ARGS, NAME, FN)                                                        \
    template <> struct KernelOf<KID> {                                                         \
        using Args = ARGS;                                                                     \
        static constexpr const char* name = NAME;                                              \
        template <bool FIN, class Wait>                                                        \
        static __device__ __forceinline__ void tile(const ARGS& a, int t, float* smem, int tid, bool live, Wait& wait) { \
            FN<FIN>(a, t, smem, tid, live, wait);                                              \
        }                                                                                      \
    };
NG_KERNEL0(KID_GAP, GapArgs, "global_avgpool", global_avgpool_tile)
NG_KERNEL0(KID_DW_LDS, DwArgs, "dwconv_lds", dwconv_lds_tile)
NG_KERNEL0(KID_FC_GEMV, FcArgs, "fc_gemv", fc_gemv_tile)
NG_KERNEL0(KID_CHANNEL_SUM, EltGradArgs, "channel_sum", channel_sum_tile)
NG_KERNEL0(KID_DW_DGRAD, DwGradArgs, "dwconv_dgrad", dw_dgrad_tile)
NG_KERNEL0(KID_DW_DGRAD_LDS, DwGradArgs, "dwconv_dgrad_lds", dw_dgrad_lds_tile)
NG_KERNEL0(KID_DW_WGRAD, DwGradArgs, "dwconv_wgrad", dw_wgrad_tile)
NG_KERNEL0(KID_POOL_DGRAD, PoolGradArgs, "pool3x3_dgrad", pool_dgrad_tile)
NG_KERNEL0(KID_POOL_DGRAD_LDS, PoolGradArgs, "pool3x3_dgrad_lds", pool_dgrad_lds_tile)
NG_KERNEL0(KID_SGD, SgdArgs, "sgd_update", sgd_tile)
NG_KERNEL0(KID_SMALL_GEMM, SmallGemmArgs, "small_gemm", small_gemm_tile)
// Two tasks in one launch (they read the same tensor and neither waits for the other): the workgroups of both are dealt
// out alternately while both have tiles left, so that the two - each bound by latency rather than by bandwidth when it runs
// alone - share the compute units from the start.
template <int KA, int KB, bool FIN, class Wait>
__device__ __forceinline__ void pair_tile(const PairArgs<typename KernelOf<KA>::Args, typename KernelOf<KB>::Args>& p, int tile, float* smem,
                                          int tid, bool live, Wait& wait) {
    const int fewer = min(p.na, p.nb);
    const bool first = tile < 2 * fewer ? (tile & 1) == 0 : p.na > p.nb;
    const int t = tile < 2 * fewer ? tile >> 1 : tile - fewer;
    if (first) KernelOf<KA>::template tile<FIN>(p.a, t, smem, tid, live, wait);
    else KernelOf<KB>::template tile<FIN>(p.b, t, smem, tid, live, wait);
}
using PairDwArgs = PairArgs<DwGradArgs, DwGradArgs>;
using PairPwArgs = PairArgs<GemmArgs, GemmArgs>;
#define NG_PAIR(KID, ARGS, NAME, KA, KB)                                                       \
    template <> struct KernelOf<KID> {                                                         \
        using Args = ARGS;                                                                     \
        static constexpr const char* name = NAME;                                              \
        template <bool FIN, class Wait>                                                        \
        static __device__ __forceinline__ void tile(const ARGS& a, int t, float* smem, int tid, bool live, Wait& wait) { \
            pair_tile<KA, KB, FIN>(a, t, smem, tid, live, wait);                               \
        }                                                                                      \
    };
NG_PAIR(KID_PAIR_DW, PairDwArgs, "dwconv_dgrad+wgrad", KID_DW_DGRAD, KID_DW_WGRAD)
NG_PAIR(KID_PAIR_DW_LDS, PairDwArgs, "dwconv_dgrad_lds+wgrad", KID_DW_DGRAD_LDS, KID_DW_WGRAD)
NG_PAIR(KID_PAIR_PW16, PairPwArgs, "conv1x1_px_dgrad+wgrad_16", KID_PW_PX_DGRAD, KID_PW_WGRAD_PX)
NG_PAIR(KID_PAIR_PW32, PairPwArgs, "conv1x1_px_dgrad+wgrad_32", KID_PW_PX_DGRAD, KID_PW_WGRAD_PX2)
#undef NG_PAIR
NG_KERNEL0(KID_SGD_BATCH, SgdBatchArgs, "sgd_update_batch", sgd_batch_tile)
#undef NG_KERNEL0

// every kernel id that has a tile function
#define NG_FOR_EACH_KID(X)                                                                                              \
    X(KID_BN) X(KID_BN_V4) X(KID_BN_R64) X(KID_BN_R16) X(KID_ADD) X(KID_ADD_V4) X(KID_ADD_R64) X(KID_ADD_R16)           \
    X(KID_CONCAT) X(KID_CONCAT_V4) X(KID_POOL) X(KID_POOL_P4) X(KID_DW_K3S1_P4) X(KID_DW_K3S1) X(KID_DW_K3S2)           \
    X(KID_DW_K5S1) X(KID_DW_K5S2) X(KID_GAP) X(KID_FC_GEMV)                                                             \
    X(KID_PW_D4) X(KID_PW_D8) X(KID_PW_D16) X(KID_PW_64) X(KID_PW_V1) X(KID_PW_V2)                                      \
    X(KID_PW_V3) X(KID_PW_V4) X(KID_PW_S1) X(KID_PW_S2) X(KID_PW_S3) X(KID_PW_S4) X(KID_C3_T16S1)                       \
    X(KID_C3_T16S2) X(KID_C3_T8S1) X(KID_C3_T8S2) X(KID_C3_M1) X(KID_C3_M2)                                             \
    X(KID_C3_M3) X(KID_C3_M4)                                                                                           \
    X(KID_PW_V1A) X(KID_PW_V2A) X(KID_PW_V3A) X(KID_PW_V4A) X(KID_PW_S1A) X(KID_PW_S2A)                                 \
    X(KID_PW_S3A) X(KID_PW_S4A) X(KID_C3_M1A) X(KID_C3_M2A) X(KID_C3_M3A) X(KID_C3_M4A)                                 \
    X(KID_POOL_A) X(KID_POOL_P4A) X(KID_C3_L32) X(KID_C3_L64)                                                          \
    X(KID_C3_P64) X(KID_C3_P96) X(KID_C3_Q32) X(KID_C3_Q64) X(KID_C3_Q128) X(KID_PW_P32) X(KID_PW_P64)                    \
    X(KID_POOL_ROW_S1) X(KID_POOL_ROW_S2) X(KID_DW_LDS)                                                                               \
    X(KID_GEMM_PW_FWD) X(KID_GEMM_PW_DGRAD) X(KID_GEMM_PW_WGRAD) X(KID_GEMM_C3_FWD) X(KID_GEMM_C3_DGRAD)                \
    X(KID_GEMM_C3_WGRAD) X(KID_SMALL_GEMM) X(KID_PW_PX_FWD) X(KID_PW_PX_DGRAD) X(KID_PW_WGRAD_PX) X(KID_PW_WGRAD_PX2) X(KID_C3_WGRAD_PX) X(KID_C3_WGRAD_PX2) X(KID_BN_RAW) X(KID_BN_DGRAD) X(KID_BN_WGRAD) X(KID_RELU_DGRAD) X(KID_DW_DGRAD) X(KID_DW_DGRAD_LDS)                \
    X(KID_DW_WGRAD) X(KID_POOL_DGRAD) X(KID_POOL_DGRAD_LDS) X(KID_GAP_DGRAD) X(KID_CHANNEL_SUM) X(KID_SLICE_PAD) X(KID_SGD) X(KID_SGD_BATCH) X(KID_BN_BACKWARD) X(KID_PAIR_DW) X(KID_PAIR_DW_LDS) X(KID_PAIR_PW16) X(KID_PAIR_PW32)

// A batch-norm epilogue is written into a task's argument block by type (C3Args or PwArgs, whose `ep` fields sit at
// different offsets): the predicates that name the type must agree with the type the kernel takes.
#define NG_CHECK_ARGS(KID)                                                                                              \
    static_assert(!has_bn_epilogue(KID) || (takes_c3_args(KID) ? std::is_base_of<C3Args, KernelOf<KID>::Args>::value    \
                                                               : std::is_base_of<PwArgs, KernelOf<KID>::Args>::value),  \
                  "takes_c3_args / has_bn_epilogue disagree with the kernel's argument type");
NG_FOR_EACH_KID(NG_CHECK_ARGS)
#undef NG_CHECK_ARGS

// Stand-alone kernel of one tile function: one workgroup per tile.
template <int KID>
__global__ __launch_bounds__(kBlock) void standalone_kernel(typename KernelOf<KID>::Args a) {
    __shared__ __align__(16) float smem[smem_floats(KID)];
    NoWait wait;
    KernelOf<KID>::template tile<false>(a, blockIdx.x, smem, threadIdx.x, true, wait);
}

// The same, with the device's clock read around it: workgroup b leaves in stamps[2 b] the time of its
// first instruction and in stamps[2 b + 1] the time at which all its stores were acknowledged (100 MHz
// constant clock; plain stores, one pair per workgroup, so the readings do not disturb each other). The
// latest end minus the earliest start is the time the GPU is busy with the task when it runs alone,
// without what the command processor spends around a dispatch.
template <int KID>
__global__ __launch_bounds__(kBlock) void timed_kernel(typename KernelOf<KID>::Args a, unsigned long long* stamps) {
    __shared__ __align__(16) float smem[smem_floats(KID)];
    unsigned long long t0 = 0;
    if (threadIdx.x == 0) t0 = wall_clock64();
    NoWait wait;
    KernelOf<KID>::template tile<false>(a, blockIdx.x, smem, threadIdx.x, true, wait);
    __builtin_amdgcn_s_waitcnt(0x0F70);                          // vmcnt(0): this wave's stores are acknowledged
    __syncthreads();
    if (threadIdx.x == 0) {
        stamps[2 * (size_t)blockIdx.x] = t0;
        stamps[2 * (size_t)blockIdx.x + 1] = wall_clock64();
    }
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
// (replay number), then dropping the compute unit's L1. A tensor that another XCD reads is
// stored and loaded with device-scope accesses, so no L2 is ever flushed or invalidated. Every wait is bounded: a workgroup that runs out of
// spins raises the error flag and every workgroup leaves.
// ------------------------------------------------------------------------------------
// One resident workgroup = kSubs sub-blocks of kBlock threads; the first `subs` of them take
// tile unit * subs + sub of every unit the workgroup owns (a task whose tiles keep the memory
// pipeline of a compute unit busy is better spread over more compute units: subs = 1). All
// sub-blocks walk the same number of units (tile functions may contain workgroup barriers):
// a sub-block without a tile calls the tile function with `live` false, which only takes
// part in the barriers.
// `words` points at the record's argument block in LDS; it is the same for every lane, so
// each word is moved into a scalar register.
template <int KID, class Wait>
__device__ __forceinline__ void run_tiles(const unsigned* words, int unit, int step, int ntiles, int subs, float* smem, int sub,
                                          int tid, bool fin, Wait& wait) {
    using A = typename KernelOf<KID>::Args;
    static_assert(sizeof(A) <= kArgWords * 4 && sizeof(A) % 4 == 0, "argument block does not fit the record");
    unsigned w[sizeof(A) / 4];
#pragma unroll
    for (size_t i = 0; i < sizeof(A) / 4; ++i) w[i] = __builtin_amdgcn_readfirstlane(words[i]);
    A a;
    __builtin_memcpy(&a, w, sizeof(A));
    const int nunits = (ntiles + subs - 1) / subs;
#define NG_LOOP(FI)                                                                  \
    for (; unit < nunits; unit += step) {                                            \
        const int tile = unit * subs + sub;                                          \
        const bool live = sub < subs && tile < ntiles;                               \
        KernelOf<KID>::template tile<FI>(a, live ? tile : 0, smem, tid, live, wait); \
    }
    if (!fin) { NG_LOOP(false) }
    else { NG_LOOP(true) }
#undef NG_LOOP
}

// The wait of one list entry for the completion counters of its parents; see NoWait for the
// contract. The first call does the work: lane j of the first wavefront polls parent j, then
// the compute unit's L1 is dropped and the workgroup meets at a barrier. Later calls (further
// tiles of the same entry) return at once.
// The polling loop of one lane.
// 0: the counter has reached the target; 1: it has not (`once`: after a single look, otherwise because
// another wait in the grid gave up); 2: ran out of spins.
__device__ __forceinline__ int spin_until(unsigned* counter, unsigned target, bool far, bool once, unsigned spin_limit,
                                                    int* error_dev, int poll_sleep) {
    unsigned spins = 0;
    for (;;) {
        unsigned seen;
        if (far) {
            seen = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            // read the counter where it lives, in this XCD's L2: a compare-and-swap that can
            // never match returns the current value (a plain load could be served by a stale
            // L1 line, and an atomic add of 0 is folded into such a load by the compiler)
            seen = 0xFFFFFFFFu;
            __hip_atomic_compare_exchange_strong(counter, &seen, 0xFFFFFFFFu, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        if ((int)(seen - target) >= 0) return 0;
        if (once) return 1;
        if (++spins > spin_limit) return 2;
        if ((spins & 63u) == 0 && __hip_atomic_load(error_dev, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return 1;
        if (poll_sleep == 0) __builtin_amdgcn_s_sleep(1);
        else if (poll_sleep == 1) __builtin_amdgcn_s_sleep(4);
        else __builtin_amdgcn_s_sleep(16);
    }
}

template <bool LATE>                 // LATE: the entry may have late parents (kernels with a fused add_n)
struct CounterWait {
    const DevPlan& plan;
    const unsigned* rec;             // the entry's record in LDS
    int* s_abort;
    int* s_late;                     // LDS flag: the late parents were already complete at the first wait
    unsigned epoch;
    int task, np, n_late, lane;      // np parents in all, the last n_late of them awaited by `late`
    unsigned long long* stamp;       // this entry's three clock readings when tracing, else nullptr (same for all lanes)
    bool pending, late_pending;
    bool far_out_;                   // the entry's results are stored with device-scope stores

    __device__ __forceinline__ bool far_out() const { return far_out_; }

    // Lane j of the first wavefront (first <= j < last) polls parent j until its counter has reached this
    // replay's target (`once`: looks a single time); true if it has. Other lanes return true.
    __device__ __forceinline__ bool poll(int first, int last, bool once) {
        bool ok = true;
        if (lane >= first && lane < last) {
            const unsigned target = rec[16 + lane] * epoch;
            const unsigned pw = rec[8 + lane];
            const bool far = (pw >> 31) != 0;
            unsigned* counter = (far ? plan.done : plan.done_near) + (size_t)(pw & 0x7fffffffu) * plan.done_stride;
            const int status = spin_until(counter, target, far, once, plan.spin_limit, plan.error_dev, plan.poll_sleep);
            ok = status == 0;
            if (status == 2) {
                atomicExch(plan.error_dev, task + 1);
                *plan.error_host = task + 1;
            }
        }
        return ok;
    }

    __device__ __forceinline__ void operator()() {
        if (!pending) return;
        pending = false;
        if (np > 0) {
            if (lane < 64) {                                    // first wavefront: lane j watches parent j
                const bool ok = poll(0, np - n_late, false);
                if (__any(!ok)) {
                    if (lane == 0) *s_abort = 1;
                }
                if (LATE && n_late > 0) {                       // usually the late parents are done as well by now
                    const bool there = poll(np - n_late, np, true);
                    const bool all_there = !__any(!there);
                    if (lane == 0) *s_late = all_there ? 1 : 0;
                }
                // Make the producers' stores visible to this compute unit. Producers on this
                // XCD have their results in the shared L2 already: dropping this CU's vector
                // L1 is enough (what a workgroup-scope acquire does when the waves of a
                // workgroup sit on different CUs). Tensors produced on another XCD are never
                // cached here at all: their loads are device-scope accesses (far_in).
                asm volatile("buffer_inv sc0" ::: "memory");
            }
            __syncthreads();                                    // also waits for the invalidate to finish
        }
        if (stamp != nullptr && lane == 0) stamp[1] = wall_clock64();
    }

    // Second wait of an entry whose tiles have a fused add_n: for the producers of the other operands.
    __device__ __forceinline__ void late() {
        if (!late_pending) return;
        late_pending = false;
        if (!LATE || n_late == 0 || *s_late != 0) return;       // same decision in every thread
        if (lane < 64) {
            const bool ok = poll(np - n_late, np, false);
            if (__any(!ok)) {
                if (lane == 0) *s_abort = 1;
            }
            asm volatile("buffer_inv sc0" ::: "memory");
        }
        __syncthreads();
    }
};

// BUILD selects which tile functions are compiled in (see in_build): the lean build leaves out the kernels
// that only large problems use - their register needs would otherwise shape the allocation of the whole
// replay kernel -, the train build has the lean kernels plus those of graphs that train.
template <int BUILD>
__global__ __launch_bounds__(kGroup) void resident_kernel(DevPlan plan, unsigned epoch) {
    constexpr int kSmemPerSub = BUILD == BUILD_FULL ? kSmemFloatsWide : kSmemFloats;
    __shared__ __align__(16) float smem_all[kSubs * kSmemPerSub];
    __shared__ uint4 recs[kRecordsInLds * (kRecordWords / 4)];
    __shared__ int s_abort, s_late;
    const int lane = threadIdx.x;
    const int sub = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kBlock), tid = (int)threadIdx.x % kBlock;
    float* smem = smem_all + sub * kSmemPerSub;
    if (lane == 0) s_abort = 0;
    const int e_begin = plan.wg_first[blockIdx.x], e_end = plan.wg_first[blockIdx.x + 1];
    // The plan keeps tensors in XCD-private L2s on the assumption that workgroups with equal index mod 8
    // share an XCD. Every launch checks it: each workgroup files its XCC id under its class together with
    // the replay number (a maximum, so whoever comes second in a class sees what the first one filed); the
    // answer is looked at when the workgroup is done, and a disagreement raises the error flag.
    unsigned long long xcc_prev = 0, xcc_mine = 0;
    if (plan.xcc_seen != nullptr && lane == 0) {
        xcc_mine = ((unsigned long long)epoch << 8) | (unsigned long long)(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 15u);   // XCC_ID, bits 3:0
        xcc_prev = __hip_atomic_fetch_max(plan.xcc_seen + (blockIdx.x & 7), xcc_mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    for (int chunk = e_begin; chunk < e_end; chunk += kRecordsInLds) {
        // this workgroup's next records: global memory -> LDS, 16 bytes per lane and load
        const int count = min(kRecordsInLds, e_end - chunk);
        __syncthreads();                                        // the previous chunk is no longer read
        {
            const uint4* src = reinterpret_cast<const uint4*>(plan.records + chunk);
            for (int i = lane; i < count * (kRecordWords / 4); i += kGroup) recs[i] = src[i];
        }
        __syncthreads();
        for (int e = 0; e < count; ++e) {
            const unsigned* rec = reinterpret_cast<const unsigned*>(recs + e * (kRecordWords / 4));
            const int task = __builtin_amdgcn_readfirstlane(rec[0]), kid = __builtin_amdgcn_readfirstlane(rec[1]);
            const int ntiles = __builtin_amdgcn_readfirstlane(rec[2]), np = __builtin_amdgcn_readfirstlane(rec[3]);
            const int tile0 = __builtin_amdgcn_readfirstlane(rec[4]), step = __builtin_amdgcn_readfirstlane(rec[5]);
            const int flags = __builtin_amdgcn_readfirstlane(rec[6]), subs_word = __builtin_amdgcn_readfirstlane(rec[7]);
            const int subs = subs_word & 0xff, xcd_peers = subs_word >> 8;
            const bool far_in = (flags & 1) != 0, far_out = (flags & 2) != 0;
            const int n_late = (flags >> 8) & 0xff;
            // tracing: thread 0 stamps the clock into this entry's own slot (plain stores, nothing waits for them)
            unsigned long long* stamp = plan.trace != nullptr ? plan.trace + 3 * (size_t)(chunk + e) : nullptr;
            if (stamp != nullptr && lane == 0) stamp[0] = wall_clock64();
            // What the task can do without its inputs (addresses, weights) happens inside the tile
            // function before it calls `wait`; an entry that fails to wait in time still runs its
            // tiles (all accesses stay in bounds) and the workgroup leaves right after.
            // (every entry has at least one round of tiles, so the tile function always gets to call the wait)
            switch (kid) {
#define NG_CASE(KID)                                                                                                         \
    case KID:                                                                                                                \
        if constexpr (in_build(BUILD, KID)) {                                                                                \
            CounterWait<has_add_epilogue(KID)> wait{plan, rec, &s_abort, &s_late, epoch, task, np, n_late, lane, stamp, true, true, far_out}; \
            run_tiles<KID>(rec + 24, tile0, step, ntiles, subs, smem, sub, tid, far_in, wait);                               \
        }                                                                                                                    \
        break;
                NG_FOR_EACH_KID(NG_CASE)
#undef NG_CASE
                default: break;
            }
            // Publish protocol, step 1: every wave waits until all of its own vector memory operations have been
            // acknowledged (stores are counted by vmcnt on this target and a store is acknowledged by the level
            // its scope names: the XCD's L2 for a plain store through the write-through L1, the memory side for
            // an sc1 store). The barrier's own workgroup-scope fence does not include this wait. Step 2: the
            // barrier - every wave of the workgroup is past step 1. Step 3 (below): one lane bumps the counter,
            // an operation issued after the barrier and therefore after every acknowledgement.
            __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0), expcnt and lgkmcnt untouched
            __syncthreads();
            if (s_abort) return;
            if (stamp != nullptr && lane == 0) stamp[2] = wall_clock64();
            if (lane == 0) {
                // Publish completion. Readers on this XCD see the data in the shared L2 and are told through
                // a counter in that same L2 (an atomic without device scope is carried out there); if there
                // are readers elsewhere the tile functions have stored through to the memory side and the
                // device-scope counter is bumped as well.
                if (flags & 4)
                    __hip_atomic_fetch_add(plan.done_near + (size_t)task * plan.done_stride, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                bool tell_device = (flags & 8) != 0;
                if (flags & 16) {
                    // two levels: count the workgroups of this XCD in its L2; only the last one goes on
                    const unsigned before = __hip_atomic_fetch_add(plan.done_xcd + ((size_t)task * 8 + (blockIdx.x & 7)) * plan.done_stride, 1u,
                                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    tell_device = before + 1u == epoch * (unsigned)xcd_peers;
                }
                if (tell_device)
                    __hip_atomic_fetch_add(plan.done + (size_t)task * plan.done_stride, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    if (plan.xcc_seen != nullptr && lane == 0 && (xcc_prev >> 8) == (xcc_mine >> 8) && (xcc_prev & 255u) != (xcc_mine & 255u)) {
        atomicExch(plan.error_dev, kErrorXcdMapping);
        *plan.error_host = kErrorXcdMapping;
    }
}

// ------------------------------------------------------------------------------------
// task construction
// ------------------------------------------------------------------------------------
template <int KID>
void set_kernel(Task& t, const typename KernelOf<KID>::Args& a, long ntiles) {
    using A = typename KernelOf<KID>::Args;
    static_assert(sizeof(A) <= kLaunchArgBytes, "argument block too large");
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

// conv1x1 forward / input gradient of a graph that trains: the kernel that reads pixels 128 bits at a time re-reads the
// activations once per 16 rows, which pays while the rows are few (the 64 x 64 LDS-staged GEMM tile otherwise).
bool pw_px_applies(const GemmArgs& a) {
    const long hw = (long)a.Ho * a.Wo;
    return hw % 4 == 0 && a.K % 4 == 0 && a.M <= 256 && a.bias == nullptr && (long)a.K * a.N * 4 < (1L << 31) &&
           (long)a.M * a.N * 4 < (1L << 31);
}
// The classifier's GEMMs (1 x 1 maps, a few thousand outputs, K up to a few hundred): no tiles. K over the lanes of a
// wavefront where both operands run along k and K is long, else a thread per output.
constexpr long kSmallGemmOutputs = 1 << 16, kSmallGemmK = 1024;
void set_small_gemm(Task& t, SmallGemmArgs a, void (*set)(Task&, const SmallGemmArgs&, long)) {
    a.by_wave = a.sak == 1 && a.sbk == 1 && a.K >= 64;
    set(t, a, a.by_wave ? ceil_div((long)a.M * a.N, kBlock / 64) : ceil_div((long)a.M * a.N, kBlock));
}
long pw_px_tiles(const GemmArgs& a) { return ceil_div(ceil_div(a.N / 4, 16) * ceil_div(a.M, 16), 4); }

// Direct conv1x1: k steps per chunk by problem depth, and the padded step count of the packed copy.
int pw_chunk(long cin) { return cin <= 64 ? 4 : (cin <= 128 ? 8 : 16); }
int pw_padded_steps(long cin) {
    const long unit = 4L * pw_chunk(cin);
    return (int)(ceil_div(ceil_div(cin, 4), unit) * unit);
}

}  // namespace

// Which XCD runs workgroup i? The planner relies on workgroups with equal i mod 8 sharing one
// (a 1-D grid is dealt out round-robin on this GPU); the runtime checks it with this probe
// before it trusts XCD-local L2s.
namespace {
__global__ __launch_bounds__(kGroup) void xcd_probe_kernel(int* xcd_of_workgroup) {
    if (threadIdx.x == 0) xcd_of_workgroup[blockIdx.x] = (int)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));   // XCC_ID, bits 3:0
}
}  // namespace
const void* xcd_probe_kernel_handle() { return reinterpret_cast<const void*>(&xcd_probe_kernel); }

// The launch that carries out the update nodes `members` (their stand-alone tasks in `tasks`) at once. The shares of
// the members are appended to `table`, the host copy of the device table that will sit at `table_dev`: the task's
// argument points at its first share there.
void make_sgd_batch_task(const std::vector<Task>& tasks, const std::vector<int>& members, std::vector<SgdTile>& table,
                         const SgdTile* table_dev, Task& t) {
    const size_t first = table.size();
    for (int v : members) {
        SgdArgs a;
        std::memcpy(&a, tasks[v].args, sizeof a);
        for (int at = 0; at < a.total || at == 0; at += kSgdTileElems)
            table.push_back(SgdTile{a.w + at, a.g + a.offset + at, at == 0 ? a.flag : nullptr, a.lr, std::min(a.total - at, kSgdTileElems)});
    }
    t = Task();
    t.block[0] = kBlock;
    set_kernel<KID_SGD_BATCH>(t, SgdBatchArgs{table_dev + first}, (long)(table.size() - first));
}

// Which two stand-alone kernels have a launch of their own together (pair_tile): input gradient first, weight gradient second.
static int pair_kid(int kid_first, int kid_second) {
    if (kid_first == KID_DW_DGRAD && kid_second == KID_DW_WGRAD) return KID_PAIR_DW;
    if (kid_first == KID_DW_DGRAD_LDS && kid_second == KID_DW_WGRAD) return KID_PAIR_DW_LDS;
    if (kid_first == KID_PW_PX_DGRAD && kid_second == KID_PW_WGRAD_PX) return KID_PAIR_PW16;
    if (kid_first == KID_PW_PX_DGRAD && kid_second == KID_PW_WGRAD_PX2) return KID_PAIR_PW32;
    return KID_NONE;
}
bool can_pair(int kid_first, int kid_second) { return pair_kid(kid_first, kid_second) != KID_NONE; }
template <int KID>
static void set_pair(const Task& first, const Task& second, Task& t) {
    typename KernelOf<KID>::Args p{};
    std::memcpy(&p.a, first.args, sizeof p.a);
    std::memcpy(&p.b, second.args, sizeof p.b);
    p.na = (int)first.ntiles, p.nb = (int)second.ntiles;
    t = Task();
    t.block[0] = kBlock;
    set_kernel<KID>(t, p, first.ntiles + second.ntiles);
}
void make_pair_task(const Task& first, const Task& second, Task& t) {
    switch (pair_kid(first.kid, second.kid)) {
        case KID_PAIR_DW: set_pair<KID_PAIR_DW>(first, second, t); break;
        case KID_PAIR_DW_LDS: set_pair<KID_PAIR_DW_LDS>(first, second, t); break;
        case KID_PAIR_PW16: set_pair<KID_PAIR_PW16>(first, second, t); break;
        case KID_PAIR_PW32: set_pair<KID_PAIR_PW32>(first, second, t); break;
        default: t = first; break;
    }
}

// The launch that computes a batch-norm's parameter gradients (task `wgrad`) and its input gradient (task `dgrad`, same
// dy, x and parameters) in one walk over dy and x.
void make_bn_backward_task(const Task& dgrad, const Task& wgrad, Task& t) {
    BnRawArgs a, d;
    std::memcpy(&a, wgrad.args, sizeof a);
    std::memcpy(&d, dgrad.args, sizeof d);
    a.dx = d.y;
    t = Task();
    t.block[0] = kBlock;
    set_kernel<KID_BN_BACKWARD>(t, a, wgrad.ntiles);
}

const void* resident_kernel_handle(int build) {
    return build == BUILD_TRAIN ? reinterpret_cast<const void*>(&resident_kernel<BUILD_TRAIN>)
                                : build == BUILD_FULL ? reinterpret_cast<const void*>(&resident_kernel<BUILD_FULL>)
                                                      : reinterpret_cast<const void*>(&resident_kernel<BUILD_LEAN>);
}

namespace {
__global__ void empty_kernel() {}
}  // namespace
const void* empty_kernel_handle() { return reinterpret_cast<const void*>(&empty_kernel); }

// The stand-alone kernel of a kernel id (nullptr if the id has none) and its name: lets the runtime
// launch a task in the variant a replay mode really executes (e.g. a convolution with its fused
// batch-norm and add_n), by itself, for timing.
const void* standalone_kernel_handle(int kid, const char** name) {
    switch (kid) {
#define NG_HANDLE(KID) \
    case KID:          \
        if (name) *name = KernelOf<KID>::name; \
        return reinterpret_cast<const void*>(&standalone_kernel<KID>);
        NG_FOR_EACH_KID(NG_HANDLE)
#undef NG_HANDLE
        default: return nullptr;
    }
}
const void* timed_kernel_handle(int kid) {
    switch (kid) {
#define NG_HANDLE(KID) \
    case KID: return reinterpret_cast<const void*>(&timed_kernel<KID>);
        NG_FOR_EACH_KID(NG_HANDLE)
#undef NG_HANDLE
        default: return nullptr;
    }
}

namespace {
// Which conv1x1 kernel a node gets. Decided from shapes alone, so that the size of the
// repacked weights is known before any memory is bound.
struct PwChoice {
    enum Kind { NONE, GEMV, LDS64, DIRECT32, K4_VEC, K4_WORD, C3_LDS, C3_PATCH, PW_PATCH } kind = NONE;
    int kid = KID_NONE;       // C3_PATCH, PW_PATCH: which of the kernels
    int in_flight = 0;        // K4: groups of 4 k-steps in flight (1..4); DIRECT32: k-steps per chunk
    int groups = 0;           // K4: groups in the packed copy (a multiple of 4 * in_flight); DIRECT32: padded k-steps
    size_t packed = 0;        // floats of repacked weights
};
// K split of the 16-row kernels: groups of 4 k-steps, padded so that every wavefront gets
// the same whole number of chunks of `in_flight` groups.
void k4_split(long k_total, long cout, PwChoice& c) {
    const long groups = ceil_div(ceil_div(k_total, 4), 4);
    long gw = ceil_div(groups, 4);                           // groups per wavefront
    if (gw <= 4) {
        c.in_flight = (int)gw;
    } else {
        const long pad3 = ceil_div(gw, 3) * 3, pad4 = ceil_div(gw, 4) * 4;
        c.in_flight = pad3 < pad4 ? 3 : 4;
        gw = std::min(pad3, pad4);
    }
    c.groups = (int)(4 * gw);
    c.packed = (size_t)((cout + 15) / 16) * c.groups * 256;
}
constexpr long kPwPatchMinCols = 2048;
constexpr long kPoolRowMinOutputs = 1 << 20;   // pool3x3: from here on the kernel with four outputs of a column per thread
constexpr long kDwLdsMinOutputs = 1 << 18;     // dwconv: from here on whole planes through LDS (dwconv_lds), where the planes allow
PwChoice choose_pw(const ng_graph* g, int v) {
    PwChoice c;
    const Node& nd = g->nodes[v];
    if (nd.op != NG_OP_CONV1X1 && nd.op != NG_OP_FC) return c;
    const Shape& o = nd.out;
    const long cin = g->nodes[nd.preds[0]].out.c;
    const long hw = o.h * o.w, cols = o.n * hw;
    if (nd.op == NG_OP_FC && o.n <= 8) { c.kind = PwChoice::GEMV; return c; }
    // many output pixels, whole blocks of 16 input channels: activations pixel-major in LDS, weights straight from memory;
    // 64-row tiles unless that leaves most compute units without one
    const long tiles64 = ((o.c + 63) / 64) * ((cols + 63) / 64);
    if (cols >= kPwPatchMinCols && cin % 16 == 0 && cin >= 64 && tiles64 >= 64 && cols * cin * 4 < (1L << 31) && !knob("NG_NO_PATCH_KERNELS")) {
        c.kind = PwChoice::PW_PATCH;
        c.kid = tiles64 < 200 ? KID_PW_P32 : KID_PW_P64;
        const long tm = c.kid == KID_PW_P32 ? 32 : 64;
        c.groups = (int)cin;
        c.packed = (size_t)cin * (size_t)((o.c + tm - 1) / tm * tm);       // [Cin / 16][CoutP][16]
        return c;
    }
    // large problems (many 64 x 64 tiles) keep the LDS-tiled throughput kernel
    if (((o.c + 63) / 64) * ((cols + 63) / 64) >= 256) {
        c.kind = PwChoice::LDS64;
        c.groups = (int)((cin + 15) / 16 * 16);                              // CinP: whole K slices of 16
        c.packed = (size_t)c.groups * (size_t)((o.c + 63) / 64 * 64);       // W^T[CinP][CoutP]
        return c;
    }
    const bool vec = hw % 4 == 0;
    const long tiles16 = ((o.c + 15) / 16) * ((cols + 15) / 16);
    if (!vec && tiles16 > 128) {                             // enough tiles anyway: 32 x 32 tiles read less
        c.kind = PwChoice::DIRECT32;
        c.in_flight = pw_chunk(cin);
        c.groups = pw_padded_steps(cin);
        c.packed = (size_t)((o.c + 15) / 16) * 64 * c.groups;
        return c;
    }
    c.kind = vec ? PwChoice::K4_VEC : PwChoice::K4_WORD;
    k4_split(cin, o.c, c);
    return c;
}
// conv3x3 with at least 8 input channels runs as an implicit GEMM with K = 9 Cin
constexpr long kC3LdsMinCols = 2048;      // measured: below this the 16 x 16 tiles (more workgroups, shorter K loops each) win
// The patch-stationary kernels: rows and pixels of a tile, pixels the patch may have.
struct PatchKernel { int kid, tm, tn, pm; };
constexpr PatchKernel kPatchKernels[] = {{KID_C3_P64, 64, 64, 256}, {KID_C3_P96, 96, 64, 256}, {KID_C3_Q32, 32, 128, 640},
                                         {KID_C3_Q64, 64, 64, 640}, {KID_C3_Q128, 64, 128, 640}};
// Largest patch a run of tn consecutive output pixels can need: the rows it touches (a run can start at the end of a
// row), stride apart, plus two, each W + 2 pad wide.
long patch_pixels(long tn, long W, long Ho, long Wo, long stride, long pad) {
    const long rows = std::min(Ho, (tn - 2) / Wo + 2);
    return ((rows - 1) * stride + 3) * (W + 2 * pad);
}
// Which patch kernel a conv3x3 gets (KID_NONE: none fits). Decided from shapes: a workgroup's time goes with the rows of
// its tile, a compute unit works its workgroups off side by side, so the estimate is (tiles per compute unit, rounded up)
// x rows; one lone workgroup per compute unit cannot keep the matrix cores busy on its own (x 1.15).
int choose_patch_kernel(const Shape& in, const Shape& out, long stride, long pad) {
    if (in.c % 16 != 0 || in.n * in.c * in.h * in.w * 4 >= (1L << 31)) return KID_NONE;
    int best = KID_NONE;
    double best_cost = 0;
    for (const PatchKernel& k : kPatchKernels) {
        if (patch_pixels(k.tn, in.w, out.h, out.w, stride, pad) > k.pm) continue;
        if ((k.tm == 32) != (out.c <= 32)) continue;                      // the 32-row kernel is for 32 output channels and fewer
        const long tiles = out.n * ceil_div(out.h * out.w, k.tn) * ceil_div(out.c, k.tm);
        const long rounds = ceil_div(tiles, 256);
        double cost = (double)rounds * k.tm * (k.tn / 64) * (rounds == 1 ? 1.15 : 1.0) * (k.pm > 256 ? 1.08 : 1.0);
        if (k.tn == 128) cost *= 0.92;                                    // the weights are fetched once for twice the pixels
        if (best == KID_NONE || cost < best_cost) best = k.kid, best_cost = cost;
    }
    return best;
}
PwChoice choose_c3(const ng_graph* g, int v) {
    PwChoice c;
    const Node& nd = g->nodes[v];
    if (nd.op != NG_OP_CONV3X3) return c;
    const Shape& in = g->nodes[nd.preds[0]].out;
    const long cin = in.c;
    if (cin < 8) return c;
    // many output pixels: the patch-stationary kernels
    if (nd.out.n * nd.out.h * nd.out.w >= kC3LdsMinCols && !knob("NG_NO_PATCH_KERNELS")) {
        const int kid = choose_patch_kernel(in, nd.out, nd.p.stride, nd.p.pad);
        for (const PatchKernel& k : kPatchKernels)
            if (k.kid == kid) {
                c.kind = PwChoice::C3_PATCH, c.kid = kid;
                c.groups = (int)cin;                                                             // CinP = Cin (a multiple of 16)
                c.packed = (size_t)(9 * cin) * (size_t)(ceil_div(nd.out.c, k.tm) * k.tm);        // [9 Cin / 16][CoutP][16]
                return c;
            }
    }
    if (nd.out.n * nd.out.h * nd.out.w >= kC3LdsMinCols) {
        c.kind = PwChoice::C3_LDS;
        const long kc = nd.out.c <= 32 ? 16 : 32, tm = nd.out.c <= 32 ? 32 : 64;     // K slice and rows per tile of the two kernels
        c.groups = (int)((cin + kc - 1) / kc * kc);                                    // CinP
        c.packed = (size_t)(9 * c.groups) * (size_t)((nd.out.c + tm - 1) / tm * tm);  // W'^T[9 CinP][CoutP]
        return c;
    }
    c.kind = PwChoice::K4_WORD;
    k4_split(9 * cin, nd.out.c, c);
    return c;
}

}  // namespace

// Floats of library-owned constant memory node v needs (repacked conv1x1 weights), 0 if none.
namespace {
// K split of a weight-gradient GEMM: enough workgroups to occupy the GPU, splits of whole K slices
void gemm_split(long m, long n, long k, int* splits, int* k_per_split) {
    const long tiles = ceil_div(m, kGemmTile) * ceil_div(n, kGemmTile);
    // A split costs its share of the K slices (about 0.5 us each) and adds one partial tile to what the workgroup
    // that arrives last has to add up (about 0.4 us each): the sum is smallest near sqrt(1.25 x slices) splits.
    const double slices = (double)ceil_div(k, 16);
    long want = (long)std::lround(std::sqrt(1.25 * slices));
    want = std::max<long>(1, std::min<long>(want, std::max<long>(1, 768 / tiles)));
    const long per = ceil_div(ceil_div(k, want), 16) * 16;
    *k_per_split = (int)per;
    *splits = (int)ceil_div(k, per);
}
// geometry of a weight-gradient node: (M, N, K) of dW[M x N] = dY[M x K] * P^T[K x N]
bool wgrad_dims(const ng_graph* g, int v, long* m, long* n, long* k) {
    const Node& nd = g->nodes[v];
    if (nd.op != NG_OP_CONV1X1_WGRAD && nd.op != NG_OP_CONV3X3_WGRAD) return false;
    const Shape& dy = g->nodes[nd.preds[0]].out;
    const Shape& x = g->nodes[nd.preds[1]].out;
    *m = dy.c, *n = x.c * (nd.op == NG_OP_CONV3X3_WGRAD ? 9 : 1), *k = dy.n * dy.h * dy.w;
    return true;
}
// Workgroups a channel of a batch-norm or depthwise parameter gradient is split over (by images): about 512 workgroups in all
long bn_wgrad_chunks(long channels, long images, long workgroups = 512) {
    const long want = std::max<long>(1, std::min<long>(images, ceil_div(workgroups, channels)));
    return ceil_div(images, ceil_div(images, want));            // no empty chunk
}
long dw_wgrad_chunks(long channels, long images) { return bn_wgrad_chunks(channels, images, knob_int("NG_DW_WGRAD_WGS", 1, 4096, 512)); }
// How a weight-gradient node is computed: which kernel, how K is split, what workspace it needs.
struct WgradPlan {
    bool px = false;              // conv1x1_wgrad_px (both operands 128 bits along the pixels) instead of the gather GEMM
    bool small = false;           // small_gemm: 1 x 1 maps and a few thousand weights (the classifier), no split, no workspace
    int block = 0;                // px: fragments of 16 x 16 weights along each side of a workgroup's block (1 or 2)
    long tiles = 0;
    int splits = 1, k_per_split = 0;
    size_t ws_floats = 0;         // partial tiles (and group sums)
    size_t cnt_words = 0;         // arrival counters behind them, a multiple of 64
};
WgradPlan wgrad_plan(const ng_graph* g, int v) {
    WgradPlan p;
    long m, n, k;
    if (!wgrad_dims(g, v, &m, &n, &k)) return p;
    const Node& nd = g->nodes[v];
    const Shape& dy = g->nodes[nd.preds[0]].out;
    const Shape& x = g->nodes[nd.preds[1]].out;
    p.tiles = ceil_div(m, kGemmTile) * ceil_div(n, kGemmTile);
    const size_t tile_floats = (size_t)kGemmTile * kGemmTile;
    if (nd.op == NG_OP_CONV1X1_WGRAD && dy.h * dy.w == 1 && m * n <= kSmallGemmOutputs && k <= kSmallGemmK) {
        p.small = true, p.splits = 1, p.k_per_split = (int)k;
        return p;
    }
    p.px = (dy.h * dy.w) % 16 == 0 && dy.elems() * 4 < (1L << 31) && x.elems() * 4 < (1L << 31) &&
           (nd.op == NG_OP_CONV1X1_WGRAD || (nd.p.stride == 1 && nd.p.pad == 1 && dy.w % 16 == 0 && dy.h == x.h && dy.w == x.w));
    const long fm = ceil_div(m, 16), fn = ceil_div(n, 16);
    p.px = p.px && fm * fn <= 256;
    if (p.px) {
        // blocks of B x B fragments of 16 x 16 weights, each split over K so that the task has about two workgroups per
        // compute unit; a wavefront wants four slices of 16 pixels at least, and the last workgroup of a block adds up
        // `splits` partial blocks
        p.block = fm * fn <= 16 ? 1 : 2;
        p.tiles = ceil_div(fm, p.block) * ceil_div(fn, p.block);
        const long most = p.block == 1 ? 64 : 32;
        const long want = std::max<long>(1, std::min<long>({ceil_div(k, 256), std::max<long>(1, 512 / p.tiles), most}));
        p.k_per_split = (int)(ceil_div(ceil_div(k, want), 64) * 64);
        p.splits = (int)ceil_div(k, p.k_per_split);
        if (p.splits > 1) {
            p.ws_floats = (size_t)p.tiles * p.splits * 256 * p.block * p.block;
            p.cnt_words = ((size_t)p.tiles + 63) & ~(size_t)63;
        }
        return p;
    }
    gemm_split(m, n, k, &p.splits, &p.k_per_split);
    if (p.splits > 1) {
        p.ws_floats = (size_t)p.tiles * p.splits * tile_floats;
        p.cnt_words = ((size_t)p.tiles + 63) & ~(size_t)63;
    }
    return p;
}
}  // namespace

size_t packed_floats(const ng_graph* g, int v) {
    const Node& nd = g->nodes[v];
    long wm, wn, wk;
    if (wgrad_dims(g, v, &wm, &wn, &wk)) {                     // split-K workspace: partial tiles, then the arrival counters
        const WgradPlan p = wgrad_plan(g, v);
        return p.ws_floats + p.cnt_words;
    }
    if (nd.op == NG_OP_DWCONV_WGRAD) {                         // per-chunk partial sums [C][chunks][K K] (padded), then one arrival counter per channel
        const Shape& x = g->nodes[nd.preds[1]].out;
        const long chunks = dw_wgrad_chunks(x.c, x.n);
        return chunks > 1 ? (size_t)((x.c * chunks * nd.p.k * nd.p.k + 63) & ~63L) + (size_t)((x.c + 63) & ~63L) : 0;
    }
    if (nd.op == NG_OP_BN_ACT_WGRAD) {                         // per-chunk sums [C][chunks][2] (padded), then one arrival counter per channel
        const Shape& x = g->nodes[nd.preds[1]].out;
        const long chunks = bn_wgrad_chunks(x.c, x.n);
        return chunks > 1 ? (size_t)((x.c * chunks * 2 + 63) & ~63L) + (size_t)((x.c + 63) & ~63L) : 0;
    }
    if (g->trainable) return 0;                                // weights change between replays: nothing is folded or repacked
    if (nd.op == NG_OP_BN_ACT) return 2 * (size_t)((nd.out.c + 3) & ~3L);   // folded scale, shift
    if (nd.op == NG_OP_CONV3X3) return choose_c3(g, v).packed;
    return choose_pw(g, v).packed;
}

// Fill node v's constant memory: one pass over the weights, at bind time.
int pack_constants(ng_graph* g, int v, float* packed, void* stream) {
    const Node& nd = g->nodes[v];
    long wm, wn, wk;
    if (wgrad_dims(g, v, &wm, &wn, &wk)) {                     // the arrival counters start at zero
        const WgradPlan p = wgrad_plan(g, v);
        if (p.cnt_words == 0) return NG_OK;
        const hipError_t e = hipMemsetAsync(packed + p.ws_floats, 0, p.cnt_words * sizeof(float), static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return g->fail(NG_EHIP, "clearing split-K counters: %s", hipGetErrorString(e));
        return NG_OK;
    }
    if (nd.op == NG_OP_DWCONV_WGRAD || nd.op == NG_OP_BN_ACT_WGRAD) {
        const size_t floats = packed_floats(g, v);
        if (floats == 0) return NG_OK;
        const size_t cnt = (size_t)((g->nodes[nd.preds[1]].out.c + 63) & ~63L);
        const hipError_t e = hipMemsetAsync(packed + floats - cnt, 0, cnt * sizeof(float), static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return g->fail(NG_EHIP, "clearing depthwise wgrad counters: %s", hipGetErrorString(e));
        return NG_OK;
    }
    if (g->trainable) return NG_OK;
    if (nd.op == NG_OP_BN_ACT) {
        for (int j = 0; j < 4; ++j)
            if (!nd.weights[j]) return g->fail(NG_EINVAL, "node %d: weight %d is a null device pointer", v, j);
        const int C = (int)nd.out.c;
        fold_bn_kernel<<<dim3((unsigned)((C + kBlock - 1) / kBlock)), dim3(kBlock), 0, static_cast<hipStream_t>(stream)>>>(
            static_cast<const float*>(nd.weights[0]), static_cast<const float*>(nd.weights[1]),
            static_cast<const float*>(nd.weights[2]), static_cast<const float*>(nd.weights[3]), nd.p.eps, packed,
            packed + ((C + 3) & ~3), C);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return g->fail(NG_EHIP, "folding batch-norm parameters: %s", hipGetErrorString(e));
        return NG_OK;
    }
    const bool c3 = nd.op == NG_OP_CONV3X3;
    const PwChoice c = c3 ? choose_c3(g, v) : choose_pw(g, v);
    if (c.packed == 0) return NG_OK;
    const int cin = (int)g->nodes[nd.preds[0]].out.c * (c3 ? 9 : 1), cout = (int)nd.out.c;
    if (!nd.weights[0]) return g->fail(NG_EINVAL, "node %d: weight 0 is a null device pointer", v);
    const dim3 grid((unsigned)((c.packed + kBlock - 1) / kBlock)), block(kBlock);
    if (c.kind == PwChoice::PW_PATCH)
        pack_pw_patch_weights_kernel<<<grid, block, 0, static_cast<hipStream_t>(stream)>>>(
            static_cast<const float*>(nd.weights[0]), packed, cout, cin, (int)(c.packed / (size_t)c.groups), (long)c.packed);
    else if (c.kind == PwChoice::C3_PATCH)
        pack_c3_patch_weights_kernel<<<grid, block, 0, static_cast<hipStream_t>(stream)>>>(
            static_cast<const float*>(nd.weights[0]), packed, cout, cin / 9, c.groups, (int)(c.packed / (9 * (size_t)c.groups)), (long)c.packed);
    else if (c.kind == PwChoice::LDS64)
        pack_pw_lds_weights_kernel<<<grid, block, 0, static_cast<hipStream_t>(stream)>>>(
            static_cast<const float*>(nd.weights[0]), packed, cout, cin, (int)(c.packed / (size_t)c.groups), (long)c.packed);
    else if (c.kind == PwChoice::C3_LDS)
        pack_c3_lds_weights_kernel<<<grid, block, 0, static_cast<hipStream_t>(stream)>>>(
            static_cast<const float*>(nd.weights[0]), packed, cout, cin / 9, c.groups, (int)(c.packed / (9 * (size_t)c.groups)), (long)c.packed);
    else if (c.kind == PwChoice::DIRECT32)
        pack_pw_weights_kernel<<<grid, block, 0, static_cast<hipStream_t>(stream)>>>(
            static_cast<const float*>(nd.weights[0]), packed, cout, cin, c.groups, (int)c.packed);
    else
        pack_pw_weights_k4_kernel<<<grid, block, 0, static_cast<hipStream_t>(stream)>>>(
            static_cast<const float*>(nd.weights[0]), packed, cout, cin, c.groups, (int)c.packed);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return g->fail(NG_EHIP, "repacking conv1x1 weights: %s", hipGetErrorString(e));
    return NG_OK;
}

int build_task(ng_graph* g, int v, char* arena, float* packed, Task& t) {
    const Node& nd = g->nodes[v];
    t = Task();
    t.block[0] = kBlock;
    if (nd.op == NG_OP_INPUT) return NG_OK;
    for (size_t j = 0; j < nd.weights.size(); ++j)
        if (!nd.weights[j] && !g->dry_run) return g->fail(NG_EINVAL, "node %d: weight %d is a null device pointer", v, (int)j);

    auto buf = [&](int id) { return reinterpret_cast<float*>(arena + g->offset[id]); };
    const Shape& o = nd.out;
    const Shape& i0 = g->nodes[nd.preds[0]].out;
    const int total = (int)o.elems();
    const int hw_out = (int)(o.h * o.w);
    auto wf = [&](int j) { return static_cast<const float*>(nd.weights[j]); };

    switch (nd.op) {
        case NG_OP_BN_ACT:
            if (g->trainable) {                                   // gamma and beta change between replays: no folded copy
                BnRawArgs a{};
                a.x = buf(nd.preds[0]), a.y = buf(v);
                a.gamma = wf(0), a.beta = wf(1), a.mean = wf(2), a.var = wf(3);
                a.eps = nd.p.eps, a.relu = nd.p.relu != 0;
                a.C = (int)o.c, a.HW = hw_out, a.N = (int)o.n, a.total = total;
                set_kernel<KID_BN_RAW>(t, a, ceil_div(total, kBlock));
                break;
            }
            [[fallthrough]];
        case NG_OP_RELU: {
            BnArgs a{};
            a.x = buf(nd.preds[0]);
            a.y = buf(v);
            if (nd.op == NG_OP_BN_ACT) {
                if (!packed) return g->fail(NG_EINVAL, "node %d: no buffer for folded batch-norm parameters", v);
                a.scale = packed, a.shift = packed + ((o.c + 3) & ~3L);
                a.relu = nd.p.relu != 0;
            } else {
                a.relu = 1;
            }
            a.C = (int)o.c, a.HW = hw_out, a.total = total;
            a.cols = (int)(o.n * hw_out);
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
            a.C = (int)o.c, a.HW = hw_out, a.cols = (int)(o.n * hw_out);
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
            // large tensors (batches): four outputs of a column per thread
            if (total >= kPoolRowMinOutputs && (nd.p.stride == 1 || nd.p.stride == 2)) {
                const long items = (long)o.n * o.c * ceil_div(o.h, 4) * o.w;
                if (nd.p.stride == 1) set_kernel<KID_POOL_ROW_S1>(t, a, ceil_div(items, kBlock));
                else set_kernel<KID_POOL_ROW_S2>(t, a, ceil_div(items, kBlock));
                break;
            }
            set_kernel<KID_POOL>(t, a, ceil_div(total, kBlock));
            break;
        }
        case NG_OP_DWCONV: {
            DwArgs a{buf(nd.preds[0]), wf(0), buf(v), (int)o.c, (int)i0.h, (int)i0.w, (int)o.h, (int)o.w, total};
            const long n = ceil_div(total, kBlock);
            // large tensors of small planes (batches): whole planes through LDS, four outputs per thread
            const long plane = (long)i0.h * i0.w, per_wg = plane <= 1024 ? 1024 / plane : 0;
            const int bd = nd.p.k / 2;
            if (total >= kDwLdsMinOutputs && (nd.p.k == 3 || nd.p.k == 5) && (nd.p.stride == 1 || nd.p.stride == 2) && i0.w % 4 == 0 &&
                o.w % 4 == 0 && per_wg > 0 && (long)o.h * o.w <= plane &&
                per_wg * (i0.h + 2 * bd) * (i0.w + 2 * bd) <= kSmemFloats) {
                a.K = nd.p.k, a.S = nd.p.stride, a.planes_per_tile = (int)per_wg;
                set_kernel<KID_DW_LDS>(t, a, ceil_div((long)o.n * o.c, per_wg));
                break;
            }
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
            if (g->trainable) {                                   // weights change between replays: read them where they are
                GemmArgs a{};
                a.a = wf(0), a.b = buf(nd.preds[0]), a.c = buf(v), a.bias = fc ? wf(1) : nullptr;
                a.M = (int)o.c, a.K = (int)i0.c, a.N = (int)(o.n * hw_out);
                a.Cin = (int)i0.c, a.Cout = (int)o.c, a.H = a.Ho = (int)o.h, a.W = a.Wo = (int)o.w, a.stride = 1;
                a.tiles_n = (int)ceil_div(a.N, kGemmTile), a.splits = 1, a.k_per_split = a.K;
                if (hw_out == 1 && (long)a.M * a.N <= kSmallGemmOutputs && a.K <= kSmallGemmK) {
                    // Y[n][o] = sum_k W[o][k] X[n][k] + b[o]
                    SmallGemmArgs sg{a.a, a.b, a.c, a.bias, a.M, a.N, a.K, a.K, 1, 1, a.K, 1, a.M, 0};
                    set_small_gemm(t, sg, [](Task& tt, const SmallGemmArgs& aa, long n) { set_kernel<KID_SMALL_GEMM>(tt, aa, n); });
                    break;
                }
                if (!fc && pw_px_applies(a)) set_kernel<KID_PW_PX_FWD>(t, a, pw_px_tiles(a));
                else set_kernel<KID_GEMM_PW_FWD>(t, a, (long)a.tiles_n * ceil_div(a.M, kGemmTile));
                break;
            }
            const PwChoice c = choose_pw(g, v);
            if (c.kind == PwChoice::GEMV) {
                FcArgs a{buf(nd.preds[0]), wf(0), wf(1), buf(v), (int)o.n, (int)i0.c, (int)o.c};
                set_kernel<KID_FC_GEMV>(t, a, ceil_div(a.Cout, kBlock / 64));
                break;
            }
            PwArgs a{};
            a.x = buf(nd.preds[0]), a.w = wf(0), a.bias = fc ? wf(1) : nullptr, a.y = buf(v);
            a.Cin = (int)i0.c, a.Cout = (int)o.c, a.HW = hw_out, a.cols = (int)(o.n * hw_out);
            if (c.kind == PwChoice::PW_PATCH) {
                if (!packed) return g->fail(NG_EINVAL, "node %d: no buffer for repacked weights", v);
                a.wp = packed, a.ksteps = c.groups;
                a.tiles_n = (int)ceil_div(a.cols, 64);
                a.mtiles = (int)ceil_div(a.Cout, c.kid == KID_PW_P32 ? 32 : 64);
                if (c.kid == KID_PW_P32) set_kernel<KID_PW_P32>(t, a, (long)a.tiles_n * a.mtiles);
                else set_kernel<KID_PW_P64>(t, a, (long)a.tiles_n * a.mtiles);
                break;
            }
            if (c.kind == PwChoice::LDS64) {
                if (!packed) return g->fail(NG_EINVAL, "node %d: no buffer for repacked weights", v);
                a.wp = packed, a.ksteps = c.groups;
                a.tiles_n = (int)ceil_div(a.cols, 64);
                set_kernel<KID_PW_64>(t, a, (long)a.tiles_n * ceil_div(a.Cout, 64));
                break;
            }
            if (!packed) return g->fail(NG_EINVAL, "node %d: no buffer for repacked weights", v);
            a.wp = packed;
            a.ksteps = c.groups;
            a.mtiles = (int)ceil_div(a.Cout, 16);
            if (c.kind == PwChoice::DIRECT32) {
                a.tiles_n = (int)ceil_div(a.cols, 32);
                const long n = (long)a.tiles_n * ceil_div(a.Cout, 32);
                if (c.in_flight == 4) set_kernel<KID_PW_D4>(t, a, n);
                else if (c.in_flight == 8) set_kernel<KID_PW_D8>(t, a, n);
                else set_kernel<KID_PW_D16>(t, a, n);
            } else if (c.kind == PwChoice::K4_VEC) {
                a.tiles_n = (int)ceil_div(a.cols, 64);
                const long n = (long)a.tiles_n * a.mtiles;
                if (c.in_flight == 1) set_kernel<KID_PW_V1>(t, a, n);
                else if (c.in_flight == 2) set_kernel<KID_PW_V2>(t, a, n);
                else if (c.in_flight == 3) set_kernel<KID_PW_V3>(t, a, n);
                else set_kernel<KID_PW_V4>(t, a, n);
            } else {
                a.tiles_n = (int)ceil_div(a.cols, 16);
                const long n = (long)a.tiles_n * a.mtiles;
                if (c.in_flight == 1) set_kernel<KID_PW_S1>(t, a, n);
                else if (c.in_flight == 2) set_kernel<KID_PW_S2>(t, a, n);
                else if (c.in_flight == 3) set_kernel<KID_PW_S3>(t, a, n);
                else set_kernel<KID_PW_S4>(t, a, n);
            }
            break;
        }
        case NG_OP_CONV3X3: {
            C3Args a{};
            a.x = buf(nd.preds[0]), a.w = wf(0), a.y = buf(v);
            a.Cin = (int)i0.c, a.Cout = (int)o.c, a.H = (int)i0.h, a.W = (int)i0.w, a.Ho = (int)o.h, a.Wo = (int)o.w;
            a.pad = nd.p.pad, a.stride = nd.p.stride;
            if (g->trainable) {
                GemmArgs ga{};
                ga.a = wf(0), ga.b = buf(nd.preds[0]), ga.c = buf(v);
                ga.M = (int)o.c, ga.K = (int)i0.c * 9, ga.N = (int)(o.n * o.h * o.w);
                ga.Cin = (int)i0.c, ga.Cout = (int)o.c, ga.H = (int)i0.h, ga.W = (int)i0.w, ga.Ho = (int)o.h, ga.Wo = (int)o.w;
                ga.stride = nd.p.stride, ga.pad = nd.p.pad;
                ga.tiles_n = (int)ceil_div(ga.N, kGemmTile), ga.splits = 1, ga.k_per_split = ga.K;
                set_kernel<KID_GEMM_C3_FWD>(t, ga, (long)ga.tiles_n * ceil_div(ga.M, kGemmTile));
                break;
            }
            const PwChoice c = choose_c3(g, v);
            if (c.kind == PwChoice::C3_PATCH) {
                if (!packed) return g->fail(NG_EINVAL, "node %d: no buffer for repacked weights", v);
                a.wp = packed, a.groups = c.groups;
                a.cols = (int)(o.n * o.h * o.w);
                for (const PatchKernel& k : kPatchKernels) {
                    if (k.kid != c.kid) continue;
                    a.tiles_xy = (int)ceil_div(o.h * o.w, k.tn);          // runs of pixels per image
                    a.tiles_n = (int)o.n * a.tiles_xy;
                    a.co_groups = (int)ceil_div(a.Cout, k.tm);
                }
                const long n = (long)a.tiles_n * a.co_groups;
                switch (c.kid) {
                    case KID_C3_P64: set_kernel<KID_C3_P64>(t, a, n); break;
                    case KID_C3_P96: set_kernel<KID_C3_P96>(t, a, n); break;
                    case KID_C3_Q32: set_kernel<KID_C3_Q32>(t, a, n); break;
                    case KID_C3_Q64: set_kernel<KID_C3_Q64>(t, a, n); break;
                    default: set_kernel<KID_C3_Q128>(t, a, n); break;
                }
                break;
            }
            if (c.kind == PwChoice::C3_LDS) {
                if (!packed) return g->fail(NG_EINVAL, "node %d: no buffer for repacked weights", v);
                a.wp = packed, a.groups = c.groups;
                a.cols = (int)(o.n * o.h * o.w);
                if (a.Cout <= 32) {
                    a.tiles_n = (int)ceil_div(a.cols, 128);
                    set_kernel<KID_C3_L32>(t, a, (long)a.tiles_n * ceil_div(a.Cout, 32));
                } else {
                    a.tiles_n = (int)ceil_div(a.cols, 64);
                    set_kernel<KID_C3_L64>(t, a, (long)a.tiles_n * ceil_div(a.Cout, 64));
                }
                break;
            }
            if (c.packed != 0) {
                if (!packed) return g->fail(NG_EINVAL, "node %d: no buffer for repacked weights", v);
                a.wp = packed, a.groups = c.groups;
                a.cols = (int)(o.n * o.h * o.w), a.tiles_n = (int)ceil_div(a.cols, 16);
                const long n = (long)a.tiles_n * ceil_div(a.Cout, 16);
                if (c.in_flight == 1) set_kernel<KID_C3_M1>(t, a, n);
                else if (c.in_flight == 2) set_kernel<KID_C3_M2>(t, a, n);
                else if (c.in_flight == 3) set_kernel<KID_C3_M3>(t, a, n);
                else set_kernel<KID_C3_M4>(t, a, n);
                break;
            }
            // small maps: 8 x 8 tiles waste fewer lanes; a stem at batch 1 (3 input channels, a large map): four times the
            // workgroups, each with a quarter of the patch to load
            const bool small = o.h * o.w <= 24 * 24 || (a.Cin <= 4 && o.n == 1);
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
        // ---- backward operators and the weight update (graphs that train) ----
        case NG_OP_CONV1X1_DGRAD:
        case NG_OP_CONV3X3_DGRAD: {
            const bool c3 = nd.op == NG_OP_CONV3X3_DGRAD;
            const Shape& dy = i0;                                 // [n][Cout][Ho][Wo]; the result has the shape of the forward input
            GemmArgs a{};
            a.a = wf(0), a.b = buf(nd.preds[0]), a.c = buf(v);
            a.Cin = (int)o.c, a.Cout = (int)dy.c, a.H = (int)o.h, a.W = (int)o.w, a.Ho = (int)dy.h, a.Wo = (int)dy.w;
            a.stride = c3 ? nd.p.stride : 1, a.pad = c3 ? nd.p.pad : 0;
            a.M = a.Cin, a.K = a.Cout * (c3 ? 9 : 1), a.N = (int)(o.n * o.h * o.w);
            a.tiles_n = (int)ceil_div(a.N, kGemmTile), a.splits = 1, a.k_per_split = a.K;
            const long n = (long)a.tiles_n * ceil_div(a.M, kGemmTile);
            if (!c3 && o.h * o.w == 1 && (long)a.M * a.N <= kSmallGemmOutputs && a.K <= kSmallGemmK) {
                // dX[n][ci] = sum_co W[co][ci] dY[n][co]
                SmallGemmArgs sg{a.a, a.b, a.c, nullptr, a.M, a.N, a.K, 1, a.M, 1, a.K, 1, a.M, 0};
                set_small_gemm(t, sg, [](Task& tt, const SmallGemmArgs& aa, long n2) { set_kernel<KID_SMALL_GEMM>(tt, aa, n2); });
                break;
            }
            if (c3) set_kernel<KID_GEMM_C3_DGRAD>(t, a, n);
            else if (pw_px_applies(a)) set_kernel<KID_PW_PX_DGRAD>(t, a, pw_px_tiles(a));
            else set_kernel<KID_GEMM_PW_DGRAD>(t, a, n);
            break;
        }
        case NG_OP_CONV1X1_WGRAD:
        case NG_OP_CONV3X3_WGRAD: {
            const bool c3 = nd.op == NG_OP_CONV3X3_WGRAD;
            const Shape& dy = i0;
            const Shape& x = g->nodes[nd.preds[1]].out;
            GemmArgs a{};
            a.a = buf(nd.preds[0]), a.b = buf(nd.preds[1]), a.c = buf(v);
            a.Cin = (int)x.c, a.Cout = (int)dy.c, a.H = (int)x.h, a.W = (int)x.w, a.Ho = (int)dy.h, a.Wo = (int)dy.w;
            a.stride = c3 ? nd.p.stride : 1, a.pad = c3 ? nd.p.pad : 0;
            a.M = a.Cout, a.N = a.Cin * (c3 ? 9 : 1), a.K = (int)(dy.n * dy.h * dy.w);
            a.tiles_n = (int)ceil_div(a.N, kGemmTile);
            const WgradPlan p = wgrad_plan(g, v);
            a.splits = p.splits, a.k_per_split = p.k_per_split;
            const long tiles = p.tiles;
            if (a.splits > 1) {
                if (!packed) return g->fail(NG_EINVAL, "node %d: no workspace for the split-K partial tiles", v);
                a.ws = packed;
                a.cnt = reinterpret_cast<unsigned*>(packed + p.ws_floats);
            }
            if (p.small) {
                // dW[co][ci] = sum_n dY[n][co] X[n][ci]
                SmallGemmArgs sg{a.a, a.b, a.c, nullptr, a.M, a.N, a.K, 1, a.M, a.N, 1, a.N, 1, 0};
                set_small_gemm(t, sg, [](Task& tt, const SmallGemmArgs& aa, long n2) { set_kernel<KID_SMALL_GEMM>(tt, aa, n2); });
                break;
            }
            if (p.px) a.tiles_n = (int)ceil_div(ceil_div(a.N, 16), p.block);
            if (p.px && c3 && p.block == 1) set_kernel<KID_C3_WGRAD_PX>(t, a, tiles * a.splits);
            else if (p.px && c3) set_kernel<KID_C3_WGRAD_PX2>(t, a, tiles * a.splits);
            else if (p.px && p.block == 1) set_kernel<KID_PW_WGRAD_PX>(t, a, tiles * a.splits);
            else if (p.px) set_kernel<KID_PW_WGRAD_PX2>(t, a, tiles * a.splits);
            else if (c3) set_kernel<KID_GEMM_C3_WGRAD>(t, a, tiles * a.splits);
            else set_kernel<KID_GEMM_PW_WGRAD>(t, a, tiles * a.splits);
            break;
        }
        case NG_OP_BN_ACT_DGRAD:
        case NG_OP_BN_ACT_WGRAD: {
            const Shape& x = g->nodes[nd.preds[1]].out;
            BnRawArgs a{};
            a.dy = buf(nd.preds[0]), a.x = buf(nd.preds[1]), a.y = buf(v);
            a.gamma = wf(0), a.beta = wf(1), a.mean = wf(2), a.var = wf(3);
            a.eps = nd.p.eps, a.relu = nd.p.relu != 0;
            a.C = (int)x.c, a.HW = (int)(x.h * x.w), a.N = (int)x.n, a.total = (int)x.elems();
            if (nd.op == NG_OP_BN_ACT_DGRAD) {
                set_kernel<KID_BN_DGRAD>(t, a, ceil_div(a.total, kBlock));
                break;
            }
            a.chunks = (int)bn_wgrad_chunks(a.C, a.N);
            if (a.chunks > 1) {
                if (!packed) return g->fail(NG_EINVAL, "node %d: no workspace for the per-chunk sums", v);
                a.ws = packed;
                a.cnt = reinterpret_cast<unsigned*>(packed + (((size_t)a.C * a.chunks * 2 + 63) & ~(size_t)63));
            }
            set_kernel<KID_BN_WGRAD>(t, a, (long)a.C * a.chunks);
            break;
        }
        case NG_OP_RELU_DGRAD:
        case NG_OP_GAP_DGRAD:
        case NG_OP_SLICE_PAD:
        case NG_OP_CHANNEL_SUM: {
            EltGradArgs a{};
            a.dy = buf(nd.preds[0]), a.x = nd.preds.size() > 1 ? buf(nd.preds[1]) : nullptr, a.y = buf(v);
            a.C = (int)o.c, a.HW = hw_out, a.N = (int)o.n, a.total = total;
            if (nd.op == NG_OP_RELU_DGRAD) {
                set_kernel<KID_RELU_DGRAD>(t, a, ceil_div(total, kBlock));
            } else if (nd.op == NG_OP_GAP_DGRAD) {
                a.scale = 1.f / (float)hw_out;
                set_kernel<KID_GAP_DGRAD>(t, a, ceil_div(total, kBlock));
            } else if (nd.op == NG_OP_SLICE_PAD) {
                a.src_C = (int)i0.c, a.src_lo = nd.p.slice_lo[0], a.cnt = nd.p.slice_hi[0] - nd.p.slice_lo[0], a.dst_lo = nd.p.slice_lo[1];
                set_kernel<KID_SLICE_PAD>(t, a, ceil_div(total, kBlock));
            } else {                                              // sums run over the input's images and pixels
                a.C = (int)i0.c, a.HW = (int)(i0.h * i0.w), a.N = (int)i0.n;
                set_kernel<KID_CHANNEL_SUM>(t, a, a.C);
            }
            break;
        }
        case NG_OP_DWCONV_DGRAD:
        case NG_OP_DWCONV_WGRAD: {
            const Shape& dy = i0;
            const Shape& x = g->nodes[nd.preds[1]].out;
            DwGradArgs a{};
            a.dy = buf(nd.preds[0]), a.x = buf(nd.preds[1]), a.y = buf(v);
            a.N = (int)x.n, a.C = (int)x.c, a.H = (int)x.h, a.W = (int)x.w, a.Ho = (int)dy.h, a.Wo = (int)dy.w;
            a.K = nd.p.k, a.S = nd.p.stride, a.total = (int)x.elems();
            if (nd.op == NG_OP_DWCONV_DGRAD) {
                a.w = wf(0);
                const long plane = (long)a.H * a.W, planes = a.total / plane;
                const int bd = a.K / 2;
                const long per_wg = plane <= 1024 ? 1024 / plane : 0;
                if ((a.K == 3 || a.K == 5) && (a.S == 1 || a.S == 2) && a.W % 4 == 0 && a.Wo % 4 == 0 && per_wg > 0 &&
                    (long)a.Ho * a.Wo <= plane && per_wg * (a.Ho + 2 * bd) * (a.Wo + 2 * bd) <= kSmemFloats) {
                    a.chunks = (int)per_wg;                        // whole planes of dx per workgroup, their dy staged in LDS
                    set_kernel<KID_DW_DGRAD_LDS>(t, a, ceil_div(planes, per_wg));
                    break;
                }
                set_kernel<KID_DW_DGRAD>(t, a, ceil_div(a.total, kBlock));
            } else {
                a.chunks = (int)dw_wgrad_chunks(a.C, a.N);
                if (a.chunks > 1) {
                    if (!packed) return g->fail(NG_EINVAL, "node %d: no workspace for the per-chunk partial sums", v);
                    a.ws = packed;
                    a.cnt = reinterpret_cast<unsigned*>(packed + (((size_t)a.C * a.chunks * a.K * a.K + 63) & ~(size_t)63));
                }
                set_kernel<KID_DW_WGRAD>(t, a, (long)a.C * a.chunks);
            }
            break;
        }
        case NG_OP_POOL_DGRAD: {
            const Shape& dy = i0;
            const Shape& x = g->nodes[nd.preds[1]].out;
            PoolGradArgs a{buf(nd.preds[0]), buf(nd.preds[1]), buf(v), (int)x.h, (int)x.w, (int)dy.h, (int)dy.w,
                           nd.p.stride, nd.p.pad, nd.p.pool_mode, (int)x.elems()};
            const long plane = (long)x.h * x.w;
            if (plane <= kPoolGradChunk && dy.h * dy.w <= plane) {      // whole planes fit a workgroup's LDS
                a.planes_per_tile = (int)(kPoolGradChunk / plane);
                set_kernel<KID_POOL_DGRAD_LDS>(t, a, ceil_div(a.total / plane, a.planes_per_tile));
            } else {
                set_kernel<KID_POOL_DGRAD>(t, a, ceil_div(a.total, kBlock));
            }
            break;
        }
        case NG_OP_SGD_UPDATE: {
            SgdArgs a{};
            a.w = const_cast<float*>(wf(0));                      // caller-owned, updated in place
            a.g = buf(nd.preds[0]), a.flag = buf(v);
            a.lr = nd.p.lr, a.offset = nd.p.slice_lo[0], a.total = nd.p.cout;
            set_kernel<KID_SGD>(t, a, ceil_div(a.total, kBlock));
            break;
        }
        default:
            return g->fail(NG_EINVAL, "node %d: operator %d has no kernel", v, nd.op);
    }
    if (t.ntiles <= 0 || t.ntiles >= (1L << 31)) return g->fail(NG_ESHAPE, "node %d: %ld tiles cannot be launched", v, t.ntiles);
    return NG_OK;
}

}  // namespace ng
