// Internal declarations shared by the host runtime and the kernel launchers.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "../../include/mtsched.h"

namespace mt {

// ---- error plumbing -------------------------------------------------------------------
int32_t fail(int32_t code, const std::string &msg);

// ---- scheduling layer (host only) ------------------------------------------------------
struct IssueItem {
    int32_t stream, tenant, op;
    int32_t mates[3] = {-1, -1, -1};   // runtime only: tenants whose operator of the same index runs in this item's launch (co-issue), -1 = none
    int32_t fuse = 0;      // runtime only: 1 = issued as part of a neighbour's launch, 2 / 3 = launches the pair (op - 1, op): depthwise + 1x1 / 1x1 + depthwise, 4 = convolution launched with the pooling operator op + 1 in its epilogue (that operator then carries 1)
};
int32_t validate_pointers(int32_t n_tenants, const int32_t *lens, int32_t n_stages, const int32_t *pointers);
void expand_pointers(int32_t n_tenants, const int32_t *lens, int32_t n_stages, const int32_t *pointers, int32_t *slices);
void stream_map(int32_t n_tenants, const int32_t *slices, int32_t concurrency, int32_t *host_stream);
std::vector<IssueItem> issue_order(int32_t n_tenants, const int32_t *slices, int32_t concurrency, int32_t order);
int32_t search_pointers(int32_t n_tenants, const int32_t *lens, const mt_search_opts *o, mt_cost_fn cost, void *user,
                        int32_t *best_pointers, double *best_cost, int32_t *rec_pointers, double *rec_cost,
                        int32_t max_records, int32_t *n_records);

int32_t playoff_pointers(int32_t n_tenants, const int32_t *lens, int32_t n_stages, const int32_t *rec_pointers,
                         const double *rec_cost, int32_t n_records, int32_t top_k, mt_cost_fn cost, void *user,
                         int32_t *best_pointers, double *best_cost, int32_t *n_evaluated);

int32_t proportional_cu_share(int32_t n_tenants, int32_t cu_count, const double *weight, int32_t *share);
int32_t search_cu_share(int32_t n_tenants, int32_t cu_count, int32_t rounds, mt_share_cost_fn cost, void *user,
                        int32_t *best_share, double *best_cost);

int32_t search_wave_priority(int32_t n_tenants, int32_t rounds, mt_share_cost_fn cost, void *user, int32_t *best_prio,
                             double *best_cost);

constexpr int IGEMM_BK = 64;   // reduction elements per implicit-GEMM tile; packed filter rows are padded to it

inline bool is_gemm_kernel(int32_t id);

// ---- kernel families -------------------------------------------------------------------
// The kernel and tile of an operator are a pure function of its shape and storage type, never of the
// stream, CU share or stage it runs in; that is what makes outputs bit-identical across schedules.
enum KernelId : int32_t {
    K_CONV_DIRECT = 0,      // one thread per output element, any shape, any storage type
    K_IGEMM_128x128 = 1,    // MFMA implicit GEMM, 128 output channels x 128 pixels per workgroup
    K_IGEMM_64x64 = 2,      // MFMA implicit GEMM, 64 x 64
    K_IGEMM_64x16 = 3,      // MFMA implicit GEMM, 64 output channels x 16 pixels (tiny-M layers, FC)
    K_DWCONV = 4,
    K_MAXPOOL = 5,
    K_AVGPOOL = 6,
    K_GAP = 7,
    K_IGEMM_128x64 = 8,     // 128 output channels x 64 pixels
    K_GEMV = 9,             // 1x1 / fully connected layers with at most 8 output pixels: weight streaming
    K_LRN = 10,             // local response normalisation across channels
    K_ADD = 11,             // element-wise sum of two tensors, activation
    K_IGEMM_PW = 12,        // 1x1 convolution on a small map: MFMA operands straight from memory, no LDS tiles
    K_STEM = 13,            // first convolution of a network (3 input channels, even horizontal stride): im2col rows straight from memory
    K_ROWB = 14,            // filter bank resident in LDS, activations straight from memory (few output channels or short reductions)
    K_PCONV = 15,           // 3x3, stride 1, padding 1: 64 x 64 implicit GEMM whose activations are staged as an input patch per 64 channels
    K_COUNT
};

inline bool is_gemm_kernel(int32_t id) {
    return id == K_IGEMM_128x128 || id == K_IGEMM_128x64 || id == K_IGEMM_64x64 || id == K_IGEMM_64x16 || id == K_GEMV ||
           id == K_IGEMM_PW;
}

// Everything a launcher needs for one operator.  Pointers are resolved per run (the first operator may
// read the caller's input buffer, the last one writes the caller's output buffer).
struct OpArgs {
    int32_t kind, kernel_id, dtype;
    int32_t N, H, W, C;          // input tensor; for a grouped convolution C is the channel count of one group
    int32_t x_ct, x_coff;        // channels per pixel of the input buffer and first channel read (x_ct == C, 0 unless grouped)
    int32_t groups;              // launches of this operator (grouped convolution), 1 otherwise
    float lrn_alpha, lrn_beta, lrn_k;
    int32_t K, R, S;             // output channels written, window
    int32_t P, Q;                // output spatial size
    int32_t sh, sw, ph, pw;
    int32_t act;
    int32_t res_ct;              // channel count of the residual tensor (0 = no residual)
    int32_t y_coff, y_ct;        // channel offset / channel count of the output tensor
    int32_t vec;                 // channels per thread of the channel-wise kernels (1, 4 or 8)
    // implicit GEMM
    int32_t gemm_k;              // R*S*C
    int32_t k_pad;               // packed weight row length (multiple of the k tile)
    int32_t n_pad;               // packed weight rows (multiple of the channel tile)
    int32_t split_k;
    int32_t wk;                  // wave groups that share an output tile (64x64 tile only): 1 or 2
    int32_t prio;                // issue priority of the kernel's waves, 0 (default) .. 3; set per launch from the schedule
    int32_t pool2;               // 1: the epilogue applies a 2x2 / stride-2 max pooling; pixels are then walked quad by quad and y is the pooled tensor
    // Exact unsigned division by Q and by P*Q without a divide (multiply-high, two shifts): n / d =
    // (t + ((n - t) >> s1)) >> s2 with t = mulhi(m, n); filled by make_divisor().
    uint32_t divq_m, divq_s1, divq_s2, divpq_m, divpq_s1, divpq_s2;
    int32_t tile_order;          // 0: channel tile fastest (an XCD shares activation tiles), 1: pixel tile fastest (shares filter tiles)
    int32_t vec_a;               // im2col gather mode: 0 element-wise, 1 16-byte chunks (C % 8 == 0), 2 tile inside one tap (C % 64 == 0)
    int32_t grid_x, grid_y, grid_z, block;
    const void *x;
    const void *w;
    const float *bias;
    const void *res;
    void *y;
    float *ws;                   // split-K partial sums
    uint32_t *counters;          // split-K arrival counters, one per output tile, zero between launches
};

// Up to four operators of different tenants that run as one launch (co-issue): workgroups with blockIdx.y == i work on
// a[i].  All of them have the same kernel, tile, split and launch shape; only their buffers differ.
constexpr int COISSUE_MAX = 4;
struct OpArgsPair {
    OpArgs a[COISSUE_MAX];
};

// Magic numbers of the division above: l = ceil(log2 d), m = floor(2^32 (2^l - d) / d) + 1, s1 = min(l, 1), s2 = max(l - 1, 0).
inline void make_divisor(uint32_t d, uint32_t &m, uint32_t &s1, uint32_t &s2) {
    uint32_t l = 0;
    while (l < 32 && ((uint64_t)1 << l) < d) ++l;
    m = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << l) - d)) / d + 1);
    s1 = l < 1 ? l : 1;
    s2 = l > 1 ? l - 1 : 0;
}

// Reduction index of the first-layer kernel (K_STEM): per filter row a run of `dummy` (1 in the aligned form, else 0) + 3 * S input elements, padded to
// `gr` groups of 8; two groups per matrix-instruction step.  The packed filter bank is ksteps x (channels / 32) x 64
// lanes x 8 elements, i.e. the operand fragments in the order the kernel reads them.
struct StemGeom {
    int dummy, seg, gr, ng, ksteps;
};
inline StemGeom stem_geom(int R, int S, int form) {
    StemGeom g;
    g.dummy = form == 1 ? 1 : 0;
    g.seg = g.dummy + 3 * S;
    g.gr = (g.seg + 7) / 8;
    g.ng = R * g.gr;
    g.ksteps = (g.ng + 1) / 2;
    return g;
}
int stem_form(int R, int S, int sw, int W, int pw, int channels);    // 0: none, 1: aligned form (one dummy element per run), 2: general form
int launch_stem(const OpArgs &a, void *stream, const OpArgs *mate = nullptr, int n_mates = 0);
// K_ROWB: waves per workgroup of the instantiation for this window / channel counts, 0 if there is none.  Its packed
// filter bank is slices x steps x tiles per slice x 64 lanes x 8 elements, a step being 16 consecutive elements of the
// (r, s, c) reduction index and a tile 32 output channels.
int rowb_waves(int R, int S, int C, int channels);
int rowb_tiles(int R, int S, int C, int channels);   // 32-channel tiles per slice of output channels (a workgroup holds one slice's filters)
// K_PCONV: patch pixels of the instantiation that holds a map of width W (0: none).  Its filter bank is [n_pad][k_pad]
// like the tile kernel's, with the reduction index ordered (64-channel chunk, tap, channel).
int pconv_patch_pixels(int W);
int launch_pconv(const OpArgs &a, void *stream, const OpArgs *mate = nullptr, int n_mates = 0);
bool rowb_patch_form(const OpArgs &a);   // 3x3, stride 1: activations staged once per tile as an input patch in LDS
int launch_rowb(const OpArgs &a, void *stream, const OpArgs *mate = nullptr, int n_mates = 0);

// Launchers (defined in the .hip files).  Return a hipError_t as int.
int launch_direct(const OpArgs &a, void *stream, const OpArgs *mate = nullptr, int n_mates = 0);
int launch_igemm(const OpArgs &a, void *stream, const OpArgs *mate = nullptr, int n_mates = 0);
// Whether the launcher of this kernel can run two operators of equal launch shape as one launch.
bool coissue_supported(const OpArgs &a);
bool dwpw_fusable(const OpArgs &dw, const OpArgs &pw);
int launch_dwpw(const OpArgs &dw, const OpArgs &pw, void *stream);   // depthwise 3x3 + the 1x1 convolution that reads it, one launch
bool pwdw_fusable(const OpArgs &pw, const OpArgs &dw);
int launch_pwdw(const OpArgs &pw, const OpArgs &dw, void *stream);   // 1x1 convolution + the depthwise 3x3 that reads it on a small map, one launch
int launch_fill_u32(uint32_t *p, size_t n, uint32_t v, void *stream);
// Device address of the library's fixed scratch array (MT_STATIC_SCRATCH_BYTES bytes) on `device`, which must be the
// current device; looked up once per device.  Returns a hipError_t as int.
int static_scratch_address(int device, void **ptr);
int launch_probe(uint32_t *out, int n_groups, void *stream);
int launch_arrive(uint32_t *counter, void *stream);                 // one thread adds 1 to *counter (system scope, release)
// Diagnostics: a register-only loop of 4 * iters 32x32x16 matrix instructions per wave (sink: n_groups * 256 floats), and
// a 16-byte grid-stride copy (mode 0) or read (mode 1; dst then holds n_groups * 256 words) of `bytes` bytes.
int launch_peak_mfma(int dtype, float *sink, int n_groups, int iters, void *stream);
int launch_peak_stream(int mode, const void *src, void *dst, size_t bytes, int n_groups, void *stream);

}  // namespace mt
