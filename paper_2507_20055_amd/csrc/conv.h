// Convolution layers in the back-substitution: geometry, device weight layouts and launchers.
//
// A convolution layer is an affine layer whose weight matrix is the expanded kernel; in the
// block-sparse picture its rows are a "Convolution block" (core = the kernel, shared by all
// positions) and the coefficient rows of a convolution layer's neurons after the first ReLU step
// are a "Patches block" (same sparsity pattern, distinct values per row; core = [rows, patch]).
// Neither dense form is ever built: kernels work on the cores.
//
// Internal neuron order of spatial layers is (H, W, C) -- channel fastest -- so that a patch
// position is a contiguous vector of channels.
#pragma once

#include "common.h"

namespace dpc {

struct ConvGeom {
    int Ci, H, W;          // input (channels, rows, columns)
    int Co, kh, kw, stride, pad;
    int Ho, Wo;            // output rows, columns
};

struct ConvWeights {
    float* core = nullptr;      // [Co][kh][kw][Ci] padded rows: row co has ld_core floats (the layer's own expressions)
    int ld_core = 0;
    float* taps = nullptr;      // [kh][kw][Co][Ci]  (transposed-convolution operand, Ci fastest)
    float* taps4 = nullptr;     // [kh][kw][Co/4][Ci][4]: the same values with four consecutive output channels innermost (Co % 4 == 0),
                                // so that a lane of the MFMA kernel fetches the four values it feeds with one 16-byte load
    float* bias_c = nullptr;    // [Co]
    ~ConvWeights();
    ConvWeights() = default;
    ConvWeights(const ConvWeights&) = delete;
    ConvWeights& operator=(const ConvWeights&) = delete;
};

void upload_conv_weights(const ConvGeom& g, const float* K /*[Co][Ci][kh][kw] host*/, const float* b, ConvWeights& out);

// Geometry of patch-form rows: row r of a pass is neuron (ho, wo, co) of the layer being bounded,
// r = (ho*rows_W + wo)*rows_C + co; its coefficients over the current layer (grid gh x gw x C) are a
// ph x pw x C patch whose top-left corner sits at grid position (ho*S - P, wo*S - P).  Positions
// outside the grid fall on zero padding and carry no neuron: their coefficients are kept at zero.
struct PatchGeom {
    int rows_W, rows_C;    // decomposition of the row index
    int ph, pw, C;         // patch extent and channels at the current layer
    int S, P;              // origin = index * S - P
    int gh, gw;            // grid (rows, columns) of the current layer
    int elems() const { return ph * pw * C; }
};

// Sign-split ReLU step + bias fold on patch-form rows (same arithmetic as the dense-row kernel;
// lambda/mu/nu are [batch, gh*gw*C] in (H,W,C) order and are gathered by patch position).
// bias_c: per-channel bias of the convolution layer below, or NULL.  shared_core: [rows_C][ld_core]
// (initial expressions: the layer's own kernel, one core per output channel) or NULL.
void launch_relax_step_patch(float* C, int ldc, double* cst, int nsides, int batch, int R, const PatchGeom& pg,
                             const float* lambda, const float* mu, const float* nu, const float* bias_c,
                             const float* shared_core, int ld_core, const float* cst_init_c, hipStream_t s);

// Concretisation of patch-form rows against per-input bounds lo, hi: [batch, gh*gw*C] (H,W,C).
void launch_concretise_patch(const float* C, int ldc, const double* cst, int nsides, int batch, int R,
                             const PatchGeom& pg, const float* lo, const float* hi, float* out_l, float* out_u,
                             const float* shared_core, int ld_core, const float* cst_init_c, hipStream_t s);

// Transposed convolution of coefficient rows through convolution layer g (one traverse iteration):
//   in : [M][ih][iw][g.Co] rows (ld_in floats apart)   -- coefficients over g's outputs
//   out: [M][oh][ow][g.Ci] rows (ld_out floats apart)  -- coefficients over g's inputs
//   out[m, y, x, ci] = sum over (ky, kx, co) with (y + off - ky) = py*stride, (x + off - kx) = px*stride,
//                      0 <= py < ih, 0 <= px < iw, of in[m, py, px, co] * K[co, ci, ky, kx].
// Dense rows: (ih, iw) = (Ho, Wo), (oh, ow) = (H, W), off = pad.  Patch rows: (oh, ow) =
// ((ih-1)*stride + kh, (iw-1)*stride + kw), off = 0.  Columns oh*ow*Ci .. ld_out-1 are zeroed.
// Returns the algorithmic flop count 2*M*ih*iw*Co*Ci*kh*kw.
double launch_conv_transpose_rows(const float* in, int64_t M, int ld_in, int ih, int iw, const ConvGeom& g,
                                  const ConvWeights& w, float* out, int ld_out, int oh, int ow, int off, hipStream_t s);

// MFMA implicit-GEMM / small-channel kernels for the same operation; false = shape not covered.
// relu != NULL: the rows are rows over the ReLU layer above g (dense rows only when g has few input channels, i.e. is
// the network's first layer) and that layer's sign-split step with the bias fold of g is applied as the rows are loaded; the row constants it adds go
// to *slots_used slots part[k * part_stride + m], k < *slots_used <= max_slots, which the consumer adds in index
// order.  Returns false, launching nothing, when the product-then-gather kernel cannot take the shape.
struct ReluOnLoad {
    const float* pk2; int ldpk;      // compact parameters (launch_pack_relax2) [batch][ldpk]
    const float* bias_c;             // bias of g per output channel
    float* part; long long part_stride; int max_slots;
    int R, batch;                    // rows are [side][input][R]
    const PatchGeom* form; int in_mod;           // patch rows: their geometry over the ReLU layer; NULL: dense rows
};
bool launch_conv_transpose_fast(const float* in, int64_t M, int ld_in, int ih, int iw, const ConvGeom& g,
                                const ConvWeights& w, float* out, int ld_out, int oh, int ow, int off, hipStream_t s,
                                const ReluOnLoad* relu = nullptr, int* slots_used = nullptr);
// Tail of a traversal of patch-form rows in one kernel: the ReLU step of the network's first ReLU layer, the
// transposed convolution through the first layer (at most 4 input channels) and the concretisation against the box
// (see conv_tail.hip).  `form` describes the rows over the ReLU layer, `conv` the first layer.  Rows are
// [side][input][R]; in: [2*batch*R][ld_in], or with shared != 0 the bounded layer's own cores [form->rows_C][ld_in]
// with constants cst_init_c.  pk2: compact ReLU parameters (launch_pack_relax2).  Returns false, launching nothing,
// when the shape is not covered.
struct PatchTail {
    const float* in; int ld_in; int shared;
    const double* cst; const float* cst_init_c;
    int R, batch;
    const PatchGeom* form; const ConvGeom* conv;
    const float* pk2; int ldpk; const float* bias_c; const float* taps;
    const float* lo; const float* hi;
    float* out_l; float* out_u;
};
bool launch_patch_tail(const PatchTail& d, hipStream_t s);

// ReuseCert through a convolution layer: G[z - z0][k][ldE] for output positions z = (input, ho, wo) in [z0, z0 + nz), rows in
// the order of the layer's split kernel matrix (see reuse.hip).  Rr: [batch][2n + 1][ldE], n = g.Ci * g.H * g.W.
void launch_reuse_gather(const float* Rr, int n, int ldE, const ConvGeom& g, int64_t z0, int64_t nz, float* G, hipStream_t s);

// Stored bounds of a convolution layer in patch form: the window of input positions a neuron's bounds reach
// (ph x pw x C0, corner of neuron (y, x) at (y*S - P, x*S - P)), ld floats per row, constant in column ph*pw*C0.
struct ReuseWindow { int ph, pw, C0, S, P, ld; };
// As launch_reuse_gather, for rows in patch form: window fi of the ReLU layer below g, window fo of g's neurons.
void launch_reuse_gather_patch(const float* Rr, int n, const ReuseWindow& fi, const ReuseWindow& fo, const ConvGeom& g, int64_t z0,
                               int64_t nz, float* G, hipStream_t s);
// Rr[b] = [lambda * L ; mu * U + nu ; unit row] as DENSE rows over the input (n0 = gh*gw*C0 columns + constant, ldE floats) from
// stored bounds in patch form (E [side][batch][n][fi.ld], or E == NULL: the shared cores [mod][ld_core] with bias [mod]);
// neuron j sits at position ((j / rows_C) / rows_W, (j / rows_C) % rows_W).
void launch_reuse_scale_expand(const float* E, const float* core, int ld_core, const float* bias, int mod, const float* lambda,
                               const float* mu, const float* nu, int batch, int n, const ReuseWindow& fi, int rows_W, int rows_C, int gh,
                               int gw, int n0, int ldE, float* Rr, hipStream_t s);

// The replacement step through a layer above rows in window form (or dense rows: the window is the image, S = P = 0) as an
// implicit contraction: E[side][(z, m)] = sum over taps and channels of the split weights A0 / A1 [M][ld_split] (lower / upper
// side, columns [part][tap][ci], bias in column 2*taps*Ci) times the rows of Rr [batch][2n+1][fi.ld], each row placed at its
// offset inside the output frame (fh x fw x C0 + constant, ld_o floats; frame_image: the whole image, else the window of the
// output position with origin index * S_o - P_o).  g describes the taps (a fully-connected layer: kh x kw = its input grid,
// one output position).  Returns the multiply-add count * 2.  reuse_window_covers: channel counts the kernel takes.
bool reuse_window_covers(int Ci);
double launch_reuse_window(const float* A0, const float* A1, int ld_split, int M, const float* Rr, int n, const ReuseWindow& fi, const ConvGeom& g,
                           int fh, int fw, int ld_o, int S_o, int P_o, bool frame_image, int batch, float* E, hipStream_t s);

int conv_algo();
int conv_half_tiles();

// Validation of certify inputs on the device.  Returns 0 = fine, 1 = lo > hi or non-finite, 2 = bad label.
// `flag` is a device int32 scratch word.  Synchronises the stream.
// Device-resident boxes and labels: copy into the result's buffers (Cc > 0: (C,H,W) -> (H,W,C)) and validate in one
// kernel; *flag must be zero before (zero_word_enqueue after a call that found an error).
void ingest_enqueue(const float* lo, const float* hi, const int32_t* label, float* l0, float* u0, int32_t* lab, int batch, int n0,
                    int Cc, int H, int W, int nK, int32_t* flag, int32_t* pinned_host_flag, hipStream_t s, float* pk = nullptr, int ld = 0);
void zero_word_enqueue(int32_t* flag, hipStream_t s);
// The same checks without waiting: the flag word lands in pinned host memory once the stream reaches the copy.
void check_inputs_enqueue(const float* lo, const float* hi, size_t count, const int32_t* label, int batch, int nK,
                          int32_t* flag, int32_t* pinned_host_flag, hipStream_t s);
int check_inputs(const float* lo, const float* hi, size_t count, const int32_t* label, int batch, int nK,
                 int32_t* flag, hipStream_t s);

}  // namespace dpc
