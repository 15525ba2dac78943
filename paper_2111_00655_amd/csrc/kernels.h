// Argument blocks and host-callable launchers of the gfx950 kernel set.
// Plain structs only, so the host-side planner can fill them without HIP
// headers.  Every launcher validates nothing: the planner (lower.cpp) is
// responsible for shapes that fit what the kernel and its grid assume.
#pragma once

#include <cstddef>
#include <cstdint>

namespace clg {

// ---- fused epilogue / prologue program ----------------------------------------------
// A short list of elementwise steps applied, in order and in registers, to
// each value a kernel produces (epilogue) or consumes (row-wise prologue).
// This is how conv+bias(+residual)+ReLU, dense+bias+GELU and longer
// elementwise tails (paper Sec. 5.5: Conv+ReLU, Conv+Add+ReLU, Add+ReLU, and
// fusions of more than ten operators) become one kernel.
constexpr int kMaxEpi = 8;

enum EpiOp : int32_t {
    EPI_NONE = 0,
    EPI_BIAS = 1,     // v += ptr[channel]
    EPI_ADD = 2,      // v += ptr[offset]           (same shape as the output)
    EPI_RELU = 3,
    EPI_GELU = 4,     // erf form
    EPI_TANH = 5,
    EPI_SCALE = 6     // v *= scalar
};

struct EpiStep {
    int32_t op;
    float scalar;
    const float *ptr;
};

struct Epilogue {
    int32_t n;
    // channel of output offset o for EPI_BIAS: (o / bias_inner) % bias_c
    int32_t bias_inner;
    int32_t bias_c;
    int32_t pad_;
    EpiStep s[kMaxEpi];
};

// The common form of a fused tail, recognised on the host: [scale] [bias]
// [residual add] [one activation], in that order.  Anything else keeps
// EF_GENERIC and is interpreted step by step.
enum EpiFastFlags : int32_t {
    EF_SCALE = 1, EF_BIAS = 2, EF_ADD = 4, EF_RELU = 8, EF_GELU = 16, EF_TANH = 32, EF_GENERIC = 64
};

struct EpiFast {
    int32_t flags;
    float scale;
    const float *bias;
    const float *add;
};

// ---- MFMA implicit GEMM ----------------------------------------------------------------
// C[i][j] = sum_k A(i,k) * B(k,j), fp32 MFMA, fp32 accumulate, epilogue in
// registers.  j is the memory-contiguous output index.
enum GemmMode : int32_t {
    GM_NT = 0,     // A[M,K] and B[N,K], both K-contiguous (dense; batch_matmul with b = [B,N,K])
    GM_NN = 1,     // A[M,K] K-contiguous, B[K,N] N-contiguous (batch_matmul with b = [B,K,N])
    GM_CONV = 2,   // A = weights [Cout, Cin*KH*KW]; B = im2col gather of x; i = cout, j = pixel
    GM_CONVT = 3   // transposed conv as stride*stride sub-pixel phases, one phase per grid.z slice
};

enum GemmTile : int32_t {
    TILE_AUTO = 0, TILE_S = 1, TILE_M = 2, TILE_L = 3, TILE_S8 = 4, TILE_S16 = 5,
    TILE_R32 = 6, TILE_R16 = 7,    // register-fed convolution kernels, 32x32 / 16x16 tiles (gemm_rf.h)
    TILE_R16X2 = 8                 // register-fed dense: a wave owns two 16x16 tiles that share the activations
};

// GemmCore is what a kernel reads on the device; GemmArgs adds the step list that the host turns into `ef`
// (or that the general kernel interprets).  A region's argument block holds cores only.
struct GemmCore {
    // The order is by who reads what: a kernel fetches its arguments with scalar loads, one cache
    // line of 64 bytes at a time, before it can do anything else, and the register-fed kernels are
    // a few microseconds long.  What they read comes first (three lines); moving the fast epilogue
    // from behind the step list to the front measured 3 % of ResNet-50's kernel time.
    // -- line 0
    const float *A;
    const float *B;
    float *C;
    float *partial;                        // split-K partial sums [splitk][numel(C)]
    int64_t c_numel;
    uint64_t rf_wo_magic;                  // floor(2^32 / WO) + 1: pixel / WO by multiply-high
    uint64_t rf_tile_magic;                // the same for rf_tile_div
    int32_t splitk, rf_tile_div;           // rf_tile_div: tiles along the fast axis of the tile order (m-tiles if rf_jmajor)
    // -- line 1
    EpiFast ef;                            // filled by launch_gemm from epi
    // convolution geometry (GM_CONV, GM_CONVT)
    int32_t Nimg, Cin, H, W, Cout, KH, KW, sh, sw, ph;
    // -- line 2
    int32_t pw, HO, WO;
    // register-fed convolution (gemm_rf.h); rf_ts = 0: not used.  A then points at the packed weights.
    int32_t rf_nch, rf_ngtot, rf_nm;       // chunks per wave, packed groups per m-tile, MFMAs per tile
    int32_t rf_jmajor, rf_groups;          // rf_groups > 1: grouped convolution (Cin, Cout are totals)
    int32_t rf_cin_tile, rf_cpg_in, rf_cpg_out;            // channels contracted per m-tile; channels per group
    int32_t M, N, K;
    int32_t lda, ldc;
    // -- line 3: dense on the register-fed kernel also reads these
    // dense only: output column n goes to (n / cs_len) * cs_stride + n % cs_len within its row block
    // (cs_len = 0: plain row-major).  This is how reshape + transpose of the result is fused (head split).
    int64_t cs_stride;
    int32_t cs_len, ldb;
    int32_t mode, tile, batch;
    int32_t rf_ts, rf_tapk, rf_wgk;        // tile edge 32|16, tap mode 1|9|4|0 (-1: dense), K-waves per workgroup
    int32_t rf_nb;                         // dense: 16-row weight tiles per wave (1, or 2 sharing the activation operand)
    int32_t rf_convt;                      // 1: transposed convolution, one sub-pixel phase per grid.z slice
    int32_t rf_d2s;                        // 1: k4 s2 p1 transposed convolution with few output channels as ONE 3x3 convolution
                                           //    over the input whose 4 * Cout rows are (channel, sub-pixel phase)
    int32_t bias_on_row;                   // 1: channel = i (conv), 0: channel = j (dense)
    int32_t gemv;                          // 1: GM_NT with at most 8 rows runs the matrix-vector kernel (a wave per column)
    int32_t patch_sz;                      // 3x3 kernel: floats per channel of the LDS input patch
    int64_t strideA, strideB, strideC;     // per batch, in elements
    // 3-D convolution on the register-fed kernels: one grid.y slice per (image, output depth);
    // the depth taps are folded into the channel index (channel' = c * KD + kd, Cin holds Cin * KD)
    int32_t D, KD, sd, pd, DO;             // input depth, depth taps, depth stride / padding, output depth (1, 1, 1, 0, 1 for 2-D)
    int32_t rf_prelu;                      // 1: relu on the input of a 2-D 1x1 convolution
    int32_t rf_fold;                       // 1: KD > 1
    int32_t rf_cs;                         // elements between two input channels (D * H * W)
    int64_t rf_img_stride;                 // elements between two images of x
    uint64_t rf_kd_magic;                  // floor(2^32 / KD) + 1
};
struct GemmArgs : GemmCore {
    Epilogue epi;
};

// Several register-fed problems of one kernel shape in one launch (a region of sibling kernels).
constexpr int kMaxRegion = 8;
struct RfMultiArgs {
    int32_t n;                             // problems, 2..kMaxRegion
    int32_t tile_end[kMaxRegion];          // problem k owns workgroups tile_end[k-1] .. tile_end[k] - 1 of grid.x
    int32_t pad_[3];
    GemmCore p[kMaxRegion];
};
// Whether `a` and `b` (both resolved for a register-fed kernel) can share a launch: same kernel
// instantiation (tile, tap mode, K-waves, geometry variant) and the same grid.y / grid.z extent.
bool rf_same_launch_shape(const GemmArgs &a, const GemmArgs &b);
// Launches the members (GemmArgs with all pointers bound and ef filled) as one kernel.
int launch_gemm_region(const GemmArgs *members, int n, void *stream);

// ---- direct convolution (any groups) and transposed convolution (any geometry) -----------------------------------------------------
struct DirectConvArgs {
    const float *x;
    const float *w;
    float *y;
    int32_t N, C, H, W, O, KH, KW, sh, sw, ph, pw, G, HO, WO;
    int32_t pro_relu;                      // relu on x first; only the depthwise kernel (G = C = O, 3x3 / 5x5 / 7x7) takes it
    int32_t transposed;                    // conv2d_transpose (w is [C][O][KH][KW], G = 1) instead of conv2d
    EpiFast ef;                            // filled by launch_direct_conv from epi
    Epilogue epi;
};
bool depthwise_fast_ok(const DirectConvArgs &a);

struct PoolArgs {
    const float *x;
    float *y;
    int32_t mode;                          // 0 max pool, 1 global average, 2 average pool (padding not counted)
    int32_t NC, H, W, KH, KW, sh, sw, ph, pw, HO, WO;
    int32_t D, KD, sd, pd, DO;             // depth axis of a 3-D window pool (1, 1, 1, 0, 1 for 2-D)
    Epilogue epi;                          // fused elementwise tail of a window pool
};

// ---- several thread-per-output problems in one launch (a region of sibling depthwise convolutions
// and window pools).  kind: 3 / 5 / 7 = depthwise convolution with that filter size (p[k].dw is read),
// 10 = max pool, 11 = average pool (p[k].pool is read); block_end is filled by the launcher.
constexpr int kMaxPlaneRegion = 8;
union PlaneMember {
    DirectConvArgs dw;
    PoolArgs pool;
};
struct PlaneMultiArgs {
    int32_t n;                             // problems, 2..kMaxPlaneRegion
    int32_t block_end[kMaxPlaneRegion];    // problem k owns workgroups block_end[k-1] .. block_end[k] - 1
    int32_t kind[kMaxPlaneRegion];
    int32_t pad_[3];
    PlaneMember p[kMaxPlaneRegion];
};
bool plane_region_pool_ok(const PoolArgs &a);
int launch_plane_region(const PlaneMultiArgs &m, void *stream);

// ---- separable convolution in one kernel (sepconv.hip) -----------------------------------------
// y = tail(Wp * dw(relu?(x))) with dw a depthwise KH x KW convolution (stride, pad) or, when wd is
// null, the plain stride-sh/sw sub-sampling of a 1x1 convolution (KH = KW = 1, pad 0).
struct SepConvArgs {
    const float *x;                        // [N][C][H][W]
    const float *wd;                       // depthwise weights [C][KH*KW], or null
    const float *wp;                       // packed 1x1 weights (sepconv_pack_bytes)
    float *y;                              // [N][Cout][HO][WO]
    int32_t N, C, H, W, Cout, KH, KW, sh, sw, ph, pw, HO, WO;
    int32_t pro_relu;                      // relu on x first
    int32_t has_dw;                        // a depthwise stage precedes the 1x1 convolution (wd is set at launch)
    int32_t ngroups, m_tiles, n_tiles, mt_per_wg, nwaves;   // set by sepconv_resolve
    EpiFast ef;                            // filled by launch_sepconv from epi; EF_GENERIC: the step list is interpreted
    Epilogue epi;
};
// The common form of a fused tail (see EpiFast) with the step operands as bound in `e`.
EpiFast make_epi_fast(const Epilogue &e);
void sepconv_resolve(SepConvArgs *a);
size_t sepconv_pack_bytes(const SepConvArgs &a);
size_t sepconv_lds_bytes(const SepConvArgs &a);
int launch_sepconv_pack(const SepConvArgs &a, const float *w, float *dst, void *stream);
int launch_sepconv(const SepConvArgs &a, void *stream);
// Several separable convolutions in one launch (a region of sibling kernels): the members share the
// kernel instantiation, i.e. sepconv_region_key (filter-size class and waves per workgroup).
constexpr int kMaxSepRegion = 4;
struct SepMultiArgs {
    int32_t n;                             // problems, 2..kMaxSepRegion
    int32_t block_end[kMaxSepRegion];      // problem k owns workgroups block_end[k-1] .. block_end[k] - 1
    int32_t pad_[3];
    SepConvArgs p[kMaxSepRegion];
};
int sepconv_region_key(const SepConvArgs &a);
int launch_sepconv_region(const SepConvArgs *members, int n, void *stream);

// ---- scaled-dot-product attention in one kernel (attention.hip) -----------------------------
// y[h] = softmax(scale * q[h] k[h]^T) v[h]; q [B][Sq][d], k and v [B][Sk][d]; y [B][Sq][d], or with
// merge = 1 the heads side by side: [Sq][B*d].
struct AttentionArgs {
    const float *q;
    const float *k;
    const float *v;
    float *y;
    int32_t B, Sq, Sk, d;
    float scale;
    int32_t merge;
};
bool attention_shape_ok(const AttentionArgs &a);       // d in {32, 64, 128}, Sk <= 512
int launch_attention(const AttentionArgs &a, void *stream);

// ---- concat: y[r][...] = x_0[r][...] x_1[r][...] ..., r < outer ---------------------------------
struct ConcatArgs {
    int32_t n;                             // operands, at most 8
    int64_t outer;                         // product of the extents before the axis
    int64_t row;                           // output elements per outer index = sum of chunk[]
    int64_t chunk[8];                      // operand elements per outer index
    const float *src[8];
    float *y;
};

// ---- row-wise reductions ------------------------------------------------------------------
struct RowwiseArgs {
    int32_t mode;                          // 0 softmax, 1 layer norm
    int32_t rows, len;
    float eps;
    const float *x;
    const float *gamma;
    const float *beta;
    float *y;
    Epilogue pro;                          // applied to x first; channel = column
    // layer norm over a sum of gathered rows (an embedding: word + position + type rows): n_gather = 2 or 3,
    // the row is ((tab[0][gid[0][r]] + tab[1][gid[1][r]]) + tab[2][gid[2][r]]), x and pro are unused.
    // Ids outside a table are clamped into it.
    int32_t n_gather;
    int32_t tab_rows[3];
    const float *tab[3];
    const int32_t *gid[3];
};

// ---- elementwise chain / gather --------------------------------------------------------------
struct EltwiseArgs {
    const float *x;                        // source tensor, or the table when ids != null
    const int32_t *ids;                    // take: row ids
    float *y;
    int64_t numel;
    int32_t row_len;                       // take: hidden size
    int32_t table_rows;                    // take: rows of the table (ids are clamped into it)
    Epilogue epi;
};

// ---- layout copy: y[o] = x[sum_d idx_d(o) * in_stride[d]] --------------------------------------
struct LayoutArgs {
    const float *x;
    float *y;
    int64_t numel;
    int32_t ndim;
    int64_t out_dims[6];
    int64_t in_strides[6];
};

// Launchers: enqueue on `stream` (a hipStream_t) and return the hipError_t
// of the launch as an int (0 = success).
int launch_gemm(const GemmArgs &a, void *stream);
int launch_direct_conv(const DirectConvArgs &a, void *stream);
int launch_pool(const PoolArgs &a, void *stream);
int launch_rowwise(const RowwiseArgs &a, void *stream);
int launch_eltwise(const EltwiseArgs &a, void *stream);
int launch_layout(const LayoutArgs &a, void *stream);
int launch_concat(const ConcatArgs &a, void *stream);
// Scratch-operand fill for the measurer: uniform values in [-1, 1) from a
// counter hash of (seed, index); row ids of a gather: uniform over [0, rows).
int launch_fill(float *p, int64_t n, uint64_t seed, void *stream);
int launch_fill_ids(int32_t *p, int64_t n, int32_t rows, uint64_t seed, void *stream);
int launch_empty(void *stream);

// Tile choice and split-K factor the GEMM launcher will use for these sizes
// (resolved at plan time so that the scratch size is known).
void gemm_resolve(GemmArgs *a, int n_cus);
size_t gemm_scratch_bytes(const GemmArgs &a);

// Register-fed convolution: decides whether the kernel runs this GM_CONV
// problem with tile edge `ts` (32 or 16) and a tail of `epi_flags`
// (EpiFastFlags); if so fills the rf_* fields and the split and returns true.
// `waves` = 1, 2, 4, 8 or 16 fixes the K-waves per workgroup; 0 lets the kernel choose (one chunk of
// MFMAs per wave, at most 16 waves); -w: as 0, but at most w waves (several chunks per wave then).
bool rf_resolve(GemmArgs *a, int ts, int epi_flags, int n_cus, int waves = 0, bool split = false);
// The same for GM_NT dense (A = activations [M,K], B = weights [N,K], no batch).
// nb = 2 (ts = 16 only): a wave computes two weight tiles against one tile of activation rows.
bool rf_resolve_dense(GemmArgs *a, int ts, int epi_flags, int n_cus, int waves = 0, int nb = 1);
// The same for GM_CONVT (kernel and output sizes divisible by the stride).
bool rf_resolve_convt(GemmArgs *a, int ts, int epi_flags, int n_cus, int waves = 0);
size_t rf_pack_bytes(const GemmArgs &a);
// Packs conv weights w [Cout][Cin][KH][KW] into dst (rf_pack_bytes) for the kernel.
int launch_rf_pack(const GemmArgs &a, const float *w, float *dst, void *stream);
int epi_fast_flags(const Epilogue &e);
// Whether the lean matrix-product kernel takes these sizes (pointer alignment aside).
bool lean_mm_shape_ok(const GemmArgs &a, int epi_flags);
// Whether the matrix-vector kernel takes these sizes (pointer alignment aside).
bool gemv_shape_ok(const GemmArgs &a, int epi_flags);

}  // namespace clg
