// Device-side records shared by the kernels and the runtime (not part of the C ABI).
#pragma once

#include <cstdint>

#include "nimble_graph.h"

namespace ng {

// One id per compiled kernel body. A task = (kernel id, argument block, number of tiles);
// a tile is the share of one 256-thread workgroup.
enum Kid : int {
    KID_NONE = 0,
    KID_BN, KID_BN_V4, KID_ADD, KID_ADD_V4, KID_CONCAT, KID_CONCAT_V4, KID_POOL,
    KID_DW_K3S1, KID_DW_K3S2, KID_DW_K5S1, KID_DW_K5S2, KID_GAP, KID_FC_GEMV,
    KID_PW_D4, KID_PW_D8, KID_PW_D16, KID_PW_64, KID_C3_T16S1, KID_C3_T16S2, KID_C3_T8S1, KID_C3_T8S2,
    // conv1x1 for small problems, K split over the wavefronts in groups of 4 k-steps, 1..4 groups in flight:
    KID_PW_V1, KID_PW_V2, KID_PW_V3, KID_PW_V4,   // 16 x 64 output tile, 128-bit activation loads (HW % 4 == 0)
    KID_PW_S1, KID_PW_S2, KID_PW_S3, KID_PW_S4,   // 16 x 16 output tile, 32-bit activation loads
    KID_BN_R64, KID_BN_R16, KID_ADD_R64, KID_ADD_R16,   // elementwise tasks on the tile grids of those two (resident replay)
    KID_C3_M1, KID_C3_M2, KID_C3_M3, KID_C3_M4,   // conv3x3 as an implicit GEMM on the matrix cores, 16 x 16 output tile
    KID_POOL_P4, KID_DW_K3S1_P4,     // windowed kernels with 4 outputs per thread (resident replay)
    // the 16-row convolutions and the pools with an add_n applied to their result before it is stored (resident replay)
    KID_PW_V1A, KID_PW_V2A, KID_PW_V3A, KID_PW_V4A, KID_PW_S1A, KID_PW_S2A, KID_PW_S3A, KID_PW_S4A,
    KID_C3_M1A, KID_C3_M2A, KID_C3_M3A, KID_C3_M4A, KID_POOL_A, KID_POOL_P4A,
    KID_C3_L32, KID_C3_L64,          // conv3x3 as an implicit GEMM staged through LDS, 32 x 128 / 64 x 64 output tiles (many columns)
    // conv3x3 for many output pixels, patch-stationary: 16 input channels of the tile's input patch sit in LDS and the nine taps
    // read it at shifted addresses; weights go from memory straight into matrix-instruction operands. Output tiles (rows x pixels)
    // 64 x 64 and 96 x 64 with a patch of up to 256 pixels; 32 x 128, 64 x 64 and 64 x 128 with up to 640 (wide images, stride 2)
    KID_C3_P64, KID_C3_P96, KID_C3_Q32, KID_C3_Q64, KID_C3_Q128,
    // conv1x1 for many output pixels on the same plan (activations pixel-major in LDS, 32 or 64 channels at a time, weights
    // straight from memory): 32 x 64 and 64 x 64 output tiles
    KID_PW_P32, KID_PW_P64,
    KID_DW_LDS,                      // depthwise 3 x 3 / 5 x 5, stride 1 / 2 on planes of up to 1024 pixels staged in LDS, four outputs side by side per thread
    KID_POOL_ROW_S1, KID_POOL_ROW_S2,   // pool3x3 for large tensors: a thread computes 4 outputs of a column, lanes run along the row (stride 1 / 2)
    // graphs that train (weights change between replays, so nothing is repacked): convolutions and fc, forward and backward,
    // as one LDS-staged MFMA GEMM that gathers its operands from the natural layouts; the other backward operators; the update
    KID_GEMM_PW_FWD, KID_GEMM_PW_DGRAD, KID_GEMM_PW_WGRAD, KID_GEMM_C3_FWD, KID_GEMM_C3_DGRAD, KID_GEMM_C3_WGRAD,
    KID_SMALL_GEMM,                  // C = A B (+ bias) of a few thousand outputs at most (the classifier of a network that trains, forward and backward): no tiles, no LDS
    KID_PW_PX_FWD, KID_PW_PX_DGRAD,  // conv1x1 forward / input gradient for few channels: pixels read 128 bits at a time straight into matrix-instruction operands (HW % 4 == 0)
    KID_C3_WGRAD_PX, KID_C3_WGRAD_PX2,  // the same for conv3x3 (stride 1, padding 1, rows of a multiple of 16 pixels): the second operand is the input shifted by the tap
    KID_PW_WGRAD_PX, KID_PW_WGRAD_PX2,  // conv1x1 weight gradient with both operands read along the pixels, 128 bits at a time (HW % 16 == 0): blocks of 16 x 16 / 32 x 32 weights
    KID_BN_RAW, KID_BN_DGRAD, KID_BN_WGRAD, KID_RELU_DGRAD, KID_DW_DGRAD, KID_DW_DGRAD_LDS, KID_DW_WGRAD, KID_POOL_DGRAD, KID_POOL_DGRAD_LDS, KID_GAP_DGRAD,
    KID_CHANNEL_SUM, KID_SLICE_PAD, KID_SGD,
    KID_SGD_BATCH,                   // several update nodes in one launch (launch-based replay modes only, in no build of the resident kernel)
    KID_BN_BACKWARD,                 // batch-norm input gradient and parameter gradients of the same (dy, x) in one launch (likewise)
    // two tasks that read the same gradient, in one launch with their workgroups interleaved (likewise): depthwise input and
    // weight gradient; conv1x1 input gradient with the weight gradient in blocks of 16 x 16 / 32 x 32
    KID_PAIR_DW, KID_PAIR_DW_LDS, KID_PAIR_PW16, KID_PAIR_PW32,
    KID_COUNT
};
constexpr bool is_train_kernel(int kid) { return kid >= KID_GEMM_PW_FWD && kid <= KID_SGD; }

// the variant without / with a fused add_n of a kernel (ids without such a variant map to themselves / KID_NONE)
constexpr int plain_variant(int kid) {
    return (kid >= KID_PW_V1A && kid <= KID_PW_S4A)
               ? kid - KID_PW_V1A + KID_PW_V1
               : (kid >= KID_C3_M1A && kid <= KID_C3_M4A) ? kid - KID_C3_M1A + KID_C3_M1
                                                          : kid == KID_POOL_A ? KID_POOL : kid == KID_POOL_P4A ? KID_POOL_P4 : kid;
}
constexpr int add_variant(int kid) {
    return (kid >= KID_PW_V1 && kid <= KID_PW_S4)
               ? kid - KID_PW_V1 + KID_PW_V1A
               : (kid >= KID_C3_M1 && kid <= KID_C3_M4) ? kid - KID_C3_M1 + KID_C3_M1A
                                                        : kid == KID_POOL ? KID_POOL_A : kid == KID_POOL_P4 ? KID_POOL_P4A : KID_NONE;
}
constexpr bool is_pool(int kid) { return plain_variant(kid) == KID_POOL || plain_variant(kid) == KID_POOL_P4; }
constexpr bool is_pw16(int kid) { return plain_variant(kid) >= KID_PW_V1 && plain_variant(kid) <= KID_PW_S4; }
constexpr bool is_c3m(int kid) { return plain_variant(kid) >= KID_C3_M1 && plain_variant(kid) <= KID_C3_M4; }
constexpr bool has_add_epilogue(int kid) { return plain_variant(kid) != kid; }
constexpr bool is_c3_patch(int kid) { return kid >= KID_C3_P64 && kid <= KID_C3_Q128; }
constexpr bool is_pw_patch(int kid) { return kid == KID_PW_P32 || kid == KID_PW_P64; }
// windowed kernels for large tensors (batches): not in the lean build, but in the full and the train build
constexpr bool is_large_tensor_kernel(int kid) { return kid == KID_POOL_ROW_S1 || kid == KID_POOL_ROW_S2 || kid == KID_DW_LDS; }
constexpr bool is_c3_lds(int kid) { return kid == KID_C3_L32 || kid == KID_C3_L64 || is_c3_patch(kid); }
// convolutions whose argument block is a C3Args (the others with a batch-norm epilogue take a PwArgs)
constexpr bool takes_c3_args(int kid) { return is_c3m(kid) || is_c3_lds(kid) || (kid >= KID_C3_T16S1 && kid <= KID_C3_T8S2); }
// kernels whose tiles can apply a batch-norm / ReLU to their results before storing them: every convolution
constexpr bool has_bn_epilogue(int kid) { return is_pw16(kid) || is_c3m(kid) || is_c3_lds(kid) || is_pw_patch(kid) || (kid >= KID_PW_D4 && kid <= KID_C3_T8S2); }

// How a kernel splits its output into tiles (see the elementwise tile functions): only tasks
// with the same partition of same-shaped outputs have matching tiles.
enum { PART_NONE = -1, PART_L256 = 0, PART_L1024 = 1, PART_R64 = 2, PART_R16 = 3 };
constexpr int partition_of(int kid_any) {
    const int kid = plain_variant(kid_any);
    return (kid == KID_BN || kid == KID_ADD || kid == KID_CONCAT || kid == KID_POOL || kid == KID_DW_K3S1 ||
            kid == KID_DW_K3S2 || kid == KID_DW_K5S1 || kid == KID_DW_K5S2)
               ? PART_L256
               : (kid == KID_BN_V4 || kid == KID_ADD_V4 || kid == KID_CONCAT_V4 || kid == KID_POOL_P4 || kid == KID_DW_K3S1_P4)
                     ? PART_L1024
                     : (kid == KID_PW_V1 || kid == KID_PW_V2 || kid == KID_PW_V3 || kid == KID_PW_V4 || kid == KID_BN_R64 || kid == KID_ADD_R64)
                           ? PART_R64
                           : (kid == KID_PW_S1 || kid == KID_PW_S2 || kid == KID_PW_S3 || kid == KID_PW_S4 || kid == KID_BN_R16 ||
                              kid == KID_ADD_R16 || kid == KID_C3_M1 || kid == KID_C3_M2 || kid == KID_C3_M3 || kid == KID_C3_M4)
                                 ? PART_R16
                                 : PART_NONE;
}

// kernels whose tiles keep a compute unit's memory pipeline or matrix cores busy for a while
constexpr bool is_matrix_kernel(int kid_any) {
    const int kid = plain_variant(kid_any);
    return (kid >= KID_PW_D4 && kid <= KID_C3_T8S2) || (kid >= KID_PW_V1 && kid <= KID_PW_S4) || (kid >= KID_C3_M1 && kid <= KID_C3_M4) ||
           kid == KID_C3_L32 || kid == KID_C3_L64 || is_c3_patch(kid) || is_pw_patch(kid);
}

// kernels of the lean build of the resident kernel: everything except the 32 x 32 and LDS-tiled
// conv1x1 and the vector-ALU conv3x3 (kernels of large problems with large register needs)
constexpr bool is_lean_kernel(int kid) {
    return (!(kid >= KID_PW_D4 && kid <= KID_C3_T8S2) || kid == KID_C3_T16S2 || kid == KID_C3_T8S2) && kid != KID_C3_L32 && kid != KID_C3_L64 && !is_c3_patch(kid) && !is_pw_patch(kid) && !is_large_tensor_kernel(kid) &&
           !is_train_kernel(kid) && !(kid >= KID_SGD_BATCH && kid <= KID_PAIR_PW32);
}
// Three builds of the resident kernel: lean (small inference problems), full (every inference kernel), train (the lean
// kernels plus the training kernels: a graph that trains runs its convolutions through the GEMM kernels, never through
// the repacked-weight kernels of the full build).
enum { BUILD_LEAN = 0, BUILD_FULL = 1, BUILD_TRAIN = 2 };
constexpr bool in_build(int build, int kid) {
    return (kid >= KID_SGD_BATCH && kid <= KID_PAIR_PW32) ? false : build == BUILD_LEAN ? is_lean_kernel(kid) : build == BUILD_FULL ? !is_train_kernel(kid) : (is_lean_kernel(kid) || is_train_kernel(kid) || is_large_tensor_kernel(kid));
}

constexpr int kBlock = 256;          // threads that work on one tile (a stand-alone kernel's workgroup)
constexpr int kSubs = 2;             // tiles a workgroup of the resident kernel works on at a time
constexpr int kGroup = kBlock * kSubs;  // threads per workgroup of the resident kernel
constexpr int kArgBytes = 256;       // size of the per-task argument block of the resident kernel's task table
constexpr int kLaunchArgBytes = 384; // size of a launched kernel's argument block (a launch of two tasks carries both blocks)

// ---- argument blocks (plain data, <= kArgBytes) ---------------------------------------
struct BnArgs {
    const float* x;
    float* y;
    const float* scale;   // [C] gamma / sqrt(var + eps), folded once at bind time; nullptr => plain ReLU
    const float* shift;   // [C] beta - mean * scale
    int relu;
    int C, HW;
    int total;            // elements
    int cols;             // 2-D partitions: columns (N * HW)
};

struct AddArgs {
    const float* x[NG_MAX_PREDS];
    float* y;
    int k;
    int total;
    int C, HW, cols;      // 2-D partitions: channels, pixels per plane, columns (N * HW)
};

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

// Optional further result of a convolution or pool tile (device-resident replay only): the add_n
// task that takes the (batch-normed) convolution result or the pooled value as one operand. The other operands come from other tasks; the tile waits for them only now (the
// entry's late parents), adds in argument order and stores. y == nullptr: none.
constexpr int kEpilogueAddMax = 4;           // operands of an add_n that can be fused
struct AddEpilogue {
    const float* x[kEpilogueAddMax - 1];     // the operands that are read, in argument order
    float* y;
    int k;                                   // operands in all, 2..kEpilogueAddMax
    int zpos;                                // argument position of the value held in registers
    int far;                                 // != 0: read the operands with device-scope loads
    int pad_;
};

struct PoolArgs {
    const float* x;
    float* y;
    int H, W, Ho, Wo;
    int stride, pad, mode;     // mode 0 max, 1 avg
    int total;                 // output elements
};

struct PoolAddArgs : PoolArgs {
    AddEpilogue ea;            // the pooled value is one operand of an add_n
};

struct DwArgs {
    const float* x;
    const float* w;            // [C][K][K]
    float* y;
    int C, H, W, Ho, Wo;
    int total;                 // output elements
    int K, S, planes_per_tile; // dwconv_lds: filter size, stride, whole (image, channel) planes per workgroup (the other kernels have K and S as template arguments)
};

struct GapArgs {
    const float* x;
    float* y;
    int HW, planes;
};

struct FcArgs {
    const float* x;            // [N][Cin]
    const float* w;            // [Cout][Cin]
    const float* b;            // [Cout]
    float* y;                  // [N][Cout]
    int N, Cin, Cout;
};

// Optional second result of a convolution tile (device-resident replay only): the batch-norm /
// ReLU task that takes over the tile partition of the convolution is applied to the values
// while they are still in registers, z = act(y * scale[c] + shift[c]) - the same arithmetic on
// the same values as the stand-alone elementwise kernel. y == nullptr: none.
struct Epilogue {
    const float* scale;        // [Cout] or nullptr (plain ReLU: scale 1, shift 0)
    const float* shift;
    float* y;                  // same shape as the convolution's result
    int relu;
};

struct PwArgs {
    const float* x;            // [N][Cin][HW]
    const float* w;            // [Cout][Cin]
    const float* bias;         // [Cout] or nullptr
    float* y;                  // [N][Cout][HW]
    int Cin, Cout, HW, cols;   // cols = N * HW
    int tiles_n;               // tiles along the column (pixel) axis
    const float* wp;           // direct kernels: weights repacked into MFMA operand order
                               // (kernels with the activations pixel-major in LDS: [Cin / 16][CoutP][16], see pack_pw_patch_weights_kernel)
    int ksteps;                // 32 x 32 kernels: k-steps of 4 in the packed copy (padded, a multiple of 4 * chunk);
                               // 16-row kernels: groups of 4 k-steps in the packed copy (a multiple of 4 * groups in flight)
    int mtiles;                // direct kernels: ceil(Cout / 16); pixel-major kernels: tiles along Cout
    Epilogue ep;
};
struct PwAddArgs : PwArgs {
    AddEpilogue ea;            // applied to the batch-normed value when ep.y is set, else to the convolution result
};

struct C3Args {
    const float* x;            // [N][Cin][H][W]
    const float* w;            // [Cout][Cin][3][3]
    float* y;                  // [N][Cout][Ho][Wo]
    int Cin, Cout, H, W, Ho, Wo;
    int pad;
    int tiles_x;               // pixel tiles along W
    int tiles_xy;              // pixel tiles per image (patch-stationary kernels: runs of consecutive pixels per image)
    int co_groups;             // channel groups (workgroups along Cout)
    // implicit-GEMM kernels: Y[Cout][cols] = W[Cout][9 Cin] * patches[9 Cin][cols]
    const float* wp;           // weights repacked into MFMA operand order, 4 k-steps per lane
                               // (patch-stationary kernels: [tap * Cin / 16 + block][CoutP][16], see pack_c3_patch_weights_kernel)
    int groups;                // groups of 4 k-steps in the packed copy (a multiple of 4 * groups in flight);
                               // LDS-staged and patch-stationary kernels: input channels of the packed copy
    int stride;
    int cols;                  // N * Ho * Wo
    int tiles_n;               // tiles along the pixel axis (patch-stationary kernels: N * tiles_xy)
    Epilogue ep;
};
struct C3AddArgs : C3Args {
    AddEpilogue ea;
};
static_assert(sizeof(PwAddArgs) <= 48 * 4 && sizeof(C3AddArgs) <= 48 * 4, "argument block the resident kernel prefetches");

// ---- training kernels -------------------------------------------------------------------
// C[M x N] = A[M x K] * B[K x N] where A, B and C are views of the convolution's natural tensors; which
// view is the kernel id's business. Cin, Cout, H, W, Ho, Wo, stride, pad describe the FORWARD convolution.
// Weight gradients have a long K (batch x pixels) and few output tiles, so K is split over `splits`
// workgroups per tile; partial tiles go to `ws`, the workgroup that arrives last (counter `cnt`) adds them
// up in split order - the result does not depend on the order of arrival.
constexpr int kGemmTile = 64;        // output tile edge
struct GemmArgs {
    const float* a;            // forward / dgrad: the weights W; wgrad: dY
    const float* b;            // forward: X; dgrad: dY; wgrad: X
    float* c;                  // forward: Y; dgrad: dX; wgrad: dW
    const float* bias;         // forward of an fc: [Cout], else nullptr
    float* ws;                 // wgrad: partial tiles [tiles][splits][64 * 64]
    unsigned* cnt;             // wgrad: arrivals per tile [tiles], zero between replays
    int M, N, K;
    int Cin, Cout, H, W, Ho, Wo, stride, pad;
    int tiles_n;               // tiles along N
    int splits, k_per_split;   // k_per_split a multiple of the K slice
    // conv1x1_wgrad_px: tiles_n = blocks of 16 B x 16 B weights along N; ws = partial blocks [blocks][splits][256 B B],
    // cnt = arrivals per block
    // conv1x1_px_fwd in the launch-based modes: a batch-norm (+ ReLU) of the result, applied while the sums are in
    // registers and stored to bn_y next to the convolution's own result (nullptr: none); parameters as they are
    const float* bn_gamma; const float* bn_beta; const float* bn_mean; const float* bn_var;
    float* bn_y;
    float bn_eps;
    int bn_relu;
};
struct BnRawArgs {             // batch-norm with its four parameter vectors as they are (they change when the graph trains)
    const float* x;            // forward input
    const float* dy;           // backward: upstream gradient (nullptr forward)
    float* y;                  // forward: output; dgrad: dx; wgrad: [2][C] = dgamma, dbeta
    const float* gamma; const float* beta; const float* mean; const float* var;
    float eps;
    int relu, C, HW, N, total;
    float* ws;                 // wgrad, chunks > 1: per-chunk sums [C][chunks][2]
    unsigned* cnt;             // wgrad, chunks > 1: arrivals per channel, zero between replays
    int chunks;                // wgrad: workgroups a channel's images are split over; dwconv_dgrad_lds: planes per workgroup
    float* dx;                 // bn_act_backward: the input gradient, written by the kernel of the parameter gradients
};
struct EltGradArgs {           // relu / global-avgpool / slice-pad / channel-sum: small elementwise backward operators
    const float* dy;
    const float* x;            // relu: forward input
    float* y;
    int C, HW, N, total;       // of the output
    int src_C, src_lo, dst_lo, cnt;   // slice-pad: dy has src_C channels; its channels [src_lo, src_lo + cnt) go to [dst_lo, dst_lo + cnt)
    float scale;               // gap: 1 / (H W)
};
struct DwGradArgs {            // depthwise backward; C, H, W, Ho, Wo, K, S of the FORWARD operator
    const float* dy; const float* x; const float* w;
    float* y;                  // dgrad: dx [N][C][H][W]; wgrad: dW [C][K][K]
    int N, C, H, W, Ho, Wo, K, S, total;
    float* ws;                 // wgrad, chunks > 1: per-chunk partial sums [C][chunks][K K]
    unsigned* cnt;             // wgrad, chunks > 1: arrivals per channel, zero between replays
    int chunks;                // wgrad: workgroups a channel's images are split over; dwconv_dgrad_lds: planes per workgroup
};
struct PoolGradArgs {          // pool backward; geometry of the FORWARD operator
    const float* dy; const float* x;
    float* y;                  // dx
    int H, W, Ho, Wo, stride, pad, mode, total;
    int planes_per_tile;       // pool3x3_dgrad_lds: whole (image, channel) planes a workgroup stages in LDS (planes_per_tile H W <= kPoolGradChunk)
};
// C[m][n] = sum_k A[m][k] B[k][n] (+ bias[m]) with every operand addressed by two strides (in floats)
struct SmallGemmArgs {
    const float* a; const float* b; float* c; const float* bias;
    int M, N, K;
    int sam, sak, sbk, sbn, scm, scn;
    int by_wave;               // 1: one wavefront per output, K over the lanes (both operands contiguous along k); 0: one thread per output
};
constexpr int kPoolGradChunk = 1024;
struct SgdArgs {
    float* w;                  // updated in place
    const float* g;            // gradient tensor; element i of w pairs with g[offset + i]
    float* flag;               // the node's own (1-element) output
    float lr;
    int offset, total;
};

// One workgroup's share of a batched update: up to kSgdTileElems consecutive elements of one update node, with the
// addresses already advanced to the share's first element. A table of these in device memory is the whole
// description of the launch.
constexpr int kSgdTileElems = 1024;
struct SgdTile {
    float* w;
    const float* g;
    float* flag;               // the node's (1-element) output if this is the node's first share, else nullptr
    float lr;
    int count;
};
struct SgdBatchArgs {
    const SgdTile* tiles;      // [ntiles]
};

// Two tasks in one launch: tiles of both, dealt out alternately while both have tiles left.
template <class A, class B>
struct PairArgs {
    A a;
    B b;
    int na, nb;                // tiles of the first and of the second task
};

// ---- device-resident replay: the task schedule as data in device memory -------------------
constexpr int kArgWords = 48;        // words of the argument block the resident kernel prefetches

struct DevTask {
    int kid;
    int ntiles;
    int n_parents;
    // 1: some reader of the output sits on another XCD, so the output is stored with
    // device-scope (memory-side) stores; 0: all readers share this task's L2.
    int release_far;
    int parent[NG_MAX_PREDS];        // tasks whose completion this task waits for
    unsigned need[NG_MAX_PREDS];     // completions parent j publishes per replay
    // != 0: some operand was produced on another XCD; all activations of this task are then
    // read with device-scope (memory-side) loads, and every producer of an operand stores
    // with device-scope stores (so no operand has dirty lines in an XCD-private L2)
    unsigned far_in;
    // which completion counters the task bumps: bit 0 the one in its XCD's L2 (waiters on the
    // same XCD), bit 1 the device-scope one (waiters elsewhere, or the task runs on several XCDs),
    // bit 2 with bit 1: in two levels (per XCD, then device scope)
    unsigned publish;
    unsigned parent_far;             // bit j: parent j is awaited through its device-scope counter
    unsigned n_late;                 // the last n_late parents are awaited inside the tile function (operands of a fused add_n)
    alignas(16) unsigned char args[kArgBytes];
};

struct DevEntry {                    // one task in one workgroup's list; tiles are counted in units of `subs`
    int task;
    int tile_begin;
    int tile_step;
    int subs;                        // sub-blocks of the workgroup that take a tile each per round (1..kSubs)
    int xcd_peers;                   // two-level completion: workgroups of this task on this workgroup's XCD, else 0
};

// What the resident kernel reads: one self-contained record per (workgroup, task) entry, the
// records of one workgroup contiguous, so that a workgroup copies its whole list into LDS
// with coalesced loads and never waits for a task description while it runs.
constexpr int kRecordWords = 24 + kArgWords;     // 288 bytes, a multiple of 16
constexpr int kRecordsInLds = 128;               // records a workgroup holds in LDS at a time (then it reloads)
struct DevRecord {
    int task, kid, ntiles, n_parents;
    int tile_begin, tile_step;                   // in units of `subs` tiles
    int flags;                                   // bit 0: device-scope loads of activations, bit 1: device-scope stores of the result,
                                                 // bit 2 / 3: bump the XCD-local / the device-scope completion counter,
                                                 // bit 4: two-level completion - bump a per-XCD counter, the last one of the
                                                 // XCD bumps the device-scope counter (tasks spread over several XCDs),
                                                 // bits 8-15: how many of the parents (the last ones) are awaited late
    int subs;                                    // bits 0-7: sub-blocks that take a tile each per round (the others idle), 1..kSubs;
                                                 // bits 8-31: two-level completion (flags bit 4): workgroups of the task on this XCD
    int parent[NG_MAX_PREDS];                    // bit 31: wait on the parent's device-scope counter
    unsigned need[NG_MAX_PREDS];
    unsigned args[kArgWords];
};
static_assert(sizeof(DevRecord) == kRecordWords * 4 && sizeof(DevRecord) % 16 == 0, "record layout");

struct DevPlan {
    const DevRecord* records;        // concatenated per-workgroup lists, each in ascending task id
    const int* wg_first;             // [n_wg + 1] offsets into records
    unsigned* done;                  // [n_nodes] device-scope completion counters, never reset between replays
    unsigned* done_near;             // [n_nodes] completion counters that live in the L2 of the task's XCD
    unsigned* done_xcd;              // [n_nodes][8] first level of the two-level completion, one counter per XCD
    int* error_dev;                  // != 0 once any wait ran out of spins
    int* error_host;                 // same value in pinned host memory, for the host to read
    unsigned spin_limit;
    int done_stride;                 // words between two tasks' counters (spreads them over memory channels)
    int poll_sleep;                  // 0, 1, 2: back-off between two polls (1, 4, 16 sleep units)
    unsigned long long* trace;       // optional [n_entries][3]: the entry starts to wait, is past the wait, has stored its tiles (100 MHz clock)
    unsigned long long* xcc_seen;    // [8] (replay number << 8 | XCC id) last filed per workgroup class (index mod 8); nullptr: every hand-over is device scope, nothing to check
};
constexpr int kErrorXcdMapping = 0x40000000;   // error-flag value: workgroups of one class (index mod 8) ran on different XCDs

}  // namespace ng
