// Shared host-side declarations of the dpcert library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string>

#include "dpcert.h"

namespace dpc {

// ---- error plumbing: no exception crosses the C ABI -------------------------------------------
void set_error(const char* fmt, ...);
struct Fail { dpc_status code; };          // thrown internally, caught at every extern "C" entry

#define DPC_HIP(expr)                                                                      \
    do {                                                                                   \
        hipError_t e__ = (expr);                                                           \
        if (e__ != hipSuccess) {                                                           \
            dpc::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
            throw dpc::Fail{e__ == hipErrorOutOfMemory ? DPC_ENOMEM : DPC_EHIP};           \
        }                                                                                  \
    } while (0)

#define DPC_REQUIRE(cond, code, ...)                                                       \
    do {                                                                                   \
        if (!(cond)) { dpc::set_error(__VA_ARGS__); throw dpc::Fail{code}; }               \
    } while (0)

// Raises a kernel's dynamic-LDS limit.  The attribute belongs to the (kernel, device) pair, so it is applied once
// for every device the kernel is launched on (thread-safe).
void ensure_dynamic_lds(const void* kernel, int bytes);

static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
static inline int64_t ceil_div(int64_t x, int64_t m) { return (x + m - 1) / m; }

// Leading dimensions of every coefficient matrix are multiples of this many floats, so that a row
// is a whole number of 128-byte lines and the contraction's K loop needs no tail.
constexpr int kLdAlign = 32;

// ---- kernel launchers (each validates the shapes its kernel assumes before launching) ---------

// Per-ReLU-neuron relaxation from the predecessor's concrete bounds (DeepPoly ReLU transformer).
// l,u: [count]; writes lambda, mu, nu and the ReLU neuron's own bounds rl, ru: [count].
void launch_relax_params_pack(const float* l, const float* u, float* lambda, float* mu, float* nu, float* rl, float* ru,
                              const float* bias, int batch, int n, int ld, float* pk, float* pk2, hipStream_t s);
void launch_relax_params(const float* l, const float* u, float* lambda, float* mu, float* nu,
                         float* rl, float* ru, int64_t count, hipStream_t s);

// Sign-split ReLU step + bias fold on dense rows; see dpc_op_relax_step.  cst_init (optional,
// [R] float) replaces the incoming constant when shared_src is used.  lambda/mu/nu may be NULL
// together (identity relaxation: only the bias fold); bias may be NULL.
void launch_relax_step(float* C, int ldc, double* cst, int nsides, int batch, int R, int n,
                       const float* lambda, const float* mu, const float* nu, const float* bias,
                       const float* shared_src, int ld_src, const float* cst_init, hipStream_t s);

// Concretisation of dense rows against per-input bounds; see dpc_op_concretise.
void launch_concretise(const float* C, int ldc, const double* cst, int nsides, int batch, int R, int n,
                       const float* lo, const float* hi, float* out_l, float* out_u,
                       const float* shared_src, int ld_src, const float* cst_init, hipStream_t s,
                       const float* part = nullptr, int nslots = 0, int64_t part_stride = 0);

// fp32 MFMA contraction Cout = A * W; see dpc_op_contract (tile loads are predicated: no padding of
// the operands is required beyond leading dimensions that are multiples of 4).
void launch_contract(const float* A, int64_t M, int K, int lda, const float* W, int N, int ldw,
                     float* Cout, int ldc, hipStream_t s);

// `batches` contractions of equal shape in one launch: problem z reads A + z*strideA, W + z*strideW and writes
// Cout + z*strideC (strides in floats; 0 shares the operand between the problems).
void launch_contract_batched(const float* A, int64_t strideA, int64_t M, int K, int lda, const float* W, int64_t strideW, int N,
                             int ldw, float* Cout, int64_t strideC, int ldc, int batches, hipStream_t s);

// Contraction with the following traversal step fused into its epilogue.  pk: packed per-(group, column)
// parameters (pm, nm, kp, kn) as float4, [nsb][ldpk]; group g = row / R.  Stored value x*(x>=0?pm:nm)
// (when store != 0), row-constant partial sums x*(x>=0?kp:kn) written to part[slot][row], one slot per
// column tile.  Returns the number of slots written, or -1 when the fused path does not cover this call
// (nothing is launched then).
struct ContractEpilogue {
    const float* pk;
    int ldpk, R, nsb;
    float* part;
    int64_t part_stride;
    int max_slots;
    int store;
};
int launch_contract_fused(const float* A, int64_t M, int K, int lda, const float* W, int N, int ldw,
                          float* Cout, int ldc, const ContractEpilogue& e, hipStream_t s);

// Whole traversal of the rows of one fully-connected layer with the coefficient rows resident in LDS
// (fill from the layer's own weight rows through the ReLU step below, then one contraction + traversal step
// per affine layer, the last one concretising against the box).  Parameters are the packed ones of
// launch_pack_relax / launch_pack_bounds, groups = 2 * B in (side, input) order.  W of every step must have
// its rows padded with zeros to a multiple of 8.  Returns false, launching nothing, when the shape is not
// covered (panels wider than 1024 columns, too few workgroups to fill the device, ...).
struct ChainStepDesc {
    const float* W;        // [round_up(K, 8)][ldw]
    const float* pk;       // [2 * B][ldpk] float4
    int K, ldw, ldpk, store;
};
struct ChainDesc {
    const float* W0;       // [R][ldw0]: the bounded layer's own rows
    const float* bias0;    // [R]
    const float* pk0;      // [2 * B][ldpk0] float4: ReLU layer directly below
    int ldw0, ldpk0, width0;
    int R, B;
    int nsteps;
    const ChainStepDesc* steps;
    float* out_l;          // [B][R]
    float* out_u;
};
bool launch_chain(const ChainDesc& d, hipStream_t s);

// ---- ReuseCert helpers (Appendix C, ReuseCert): see reuse.hip for the layout -------------------
// Rr[b] = [lambda * L ; mu * U + nu ; unit row] from the stored bounds E[side][b][n][ldE] of the layer below the ReLU
// layer, or (E == NULL) from the first layer's shared rows (W1 [n][ldw], bias [n]).
// (mod > 0: the shared rows repeat every mod rows -- the cores of a first convolution layer, bias per channel.)
void launch_reuse_scale(const float* E, const float* W1, int ldw, const float* bias, const float* lambda, const float* mu,
                        const float* nu, int batch, int n, int n0, int ldE, float* Rr, hipStream_t s, int mod = 0);
// dst[m] = [c+ | c- | constant] (side 0) or [c- | c+ | constant] (side 1) of row m of src ([rows][ld_src], n columns);
// constant = bias_d[m] if given, else bias_f[m]; side = m / rows_per_side (rows_per_side > 0) or side0.
void launch_reuse_split(const float* src, int ld_src, const float* bias_f, const double* bias_d, int64_t rows, int n,
                        float* dst, int ld_dst, int64_t rows_per_side, int side0, hipStream_t s);
// cst[m] = C[m][col]
void launch_reuse_const(const float* C, int ldc, int col, int64_t rows, double* cst, hipStream_t s);

// pk[side][b][c] = (pm, nm, kp, kn) of the sign-split ReLU step through a ReLU layer with relaxation
// (lambda, mu, nu) followed by the bias fold of the layer below (bias may be NULL); columns n..ld-1 zero.
void launch_pack_relax(const float* lambda, const float* mu, const float* nu, const float* bias, int batch, int n,
                       int ld, float* pk, hipStream_t s);
// Split-precision contraction (experiment; see contract_split.hip).  terms = 2 ("bf16x3") or 3 ("bf16x6").
// Wt: [terms][round_up(N,128)][round_up(K,32)] bf16, built by launch_split_weights from W [K][ldw] fp32.
size_t split_weights_elems(int K, int N, int terms, int* ldk, int* npad);
void launch_split_weights(const float* W, int K, int N, int ldw, int terms, void* Wt, hipStream_t s);
void launch_contract_split(const float* A, int64_t M, int K, int lda, const void* Wt, int terms, int N, float* C, int ldc,
                           hipStream_t s);
int launch_contract_split_fused(const float* A, int64_t M, int K, int lda, const void* Wt, int terms, int N, float* C, int ldc,
                                const ContractEpilogue& e, hipStream_t s);
int contract_split_terms();

// Tuning knobs.  Process-wide values (dpc_tuning_set) can be overridden per network (dpc_network_tuning_set); the values in
// force on a thread are those of the network whose call is running on it (TuningScope), else the process-wide ones.
enum TuneKey {
    TK_CONTRACT_VARIANT, TK_CONTRACT_REMAP, TK_CONV_ALGO, TK_CONV_HALF_TILES, TK_MERGE_FINAL, TK_REUSE_PATCH, TK_REUSE_WINDOW,
    TK_REUSE_WINDOW_CK, TK_REUSE_WINDOW_TILES, TK_CHAIN, TK_CHAIN_ROWS, TK_CONTRACT_SPLIT_WIDE, TK_CONTRACT_SPLIT, TK_ROWS_PER_WAVE,
    TK_ROWS_STREAM, TK_STREAM_WGS_PER_CU, TK_COUNT
};
struct Tuning { int v[TK_COUNT]; };
int tune(TuneKey k);
struct TuningScope {
    explicit TuningScope(const Tuning* t);
    ~TuningScope();
    TuningScope(const TuningScope&) = delete;
    TuningScope& operator=(const TuningScope&) = delete;
private:
    const Tuning* prev_;
};
// dst rows += a block of the same expression that waited on a skip connection (residual networks); rows are
// [M][ph2*pw2*C] patches (dense rows: ph2 = pw2 = 1, C = n), the block is ph1 x pw1 x C at offset (d, d).
// kind 0: src[m][..]; kind 1: src[r % rows_C][..] (r = m % R); kind 2: += 1 on channel r % rows_C of position (d, d).
void launch_merge_block(float* dst, int ld_dst, int64_t M, int R, int rows_C, int ph2, int pw2, int C, int kind,
                        const float* src, int ld_src, int ph1, int pw1, int d, hipStream_t s);
// cst[m] += concretisation of a waiting block (kinds as above) against lo, hi [batch][n], the bounds of the layer
// the block is over; patch != 0: the block is a ph x pw x C patch with origin index * S - P on a gh x gw grid.
void launch_block_bound(double* cst, int64_t M, int R, int rows_C, int rows_W, int batch, int nsides, int n, int kind,
                        const float* src, int ld_src, const float* lo, const float* hi, int patch, int ph, int pw, int C, int S,
                        int P, int gh, int gw, hipStream_t s);
// Patch-form rows at the input layer -> dense rows over the input (dst zero before); see kernels_rows.hip.
void launch_expand_patch_rows(const float* src, int ld_src, int shared_mod, const double* cst_in, const float* cst_init_c,
                              int64_t M, int R, int rows_C, int rows_W, int ph, int pw, int C, int S, int P, int gh, int gw,
                              float* dst, int ld_dst, double* cst_out, hipStream_t s);
// One input's kept symbolic bounds from internal (H,W,C) row / column orders to (C,H,W); rC / cC = 0: no shape.
void launch_sym_export(const float* src, int ld_src, const double* cst, int n, int n0, int rC, int rH, int rW, int cC, int cH, int cW,
                       float* out, float* cst_out, hipStream_t s);
// rows[r][:] *= scale[r]; cst[r] = scale[r] * (bias_f ? bias_f[r] : cst[r]) + (add ? add[r] : 0).
void launch_scale_rows(float* rows, int ld, int n, int ncols, double* cst, const float* bias_f, const float* scale, const float* add,
                       hipStream_t s);
void launch_add_vectors(const float* a, const float* b, float* out, int64_t n, hipStream_t s);
void launch_fold_slots(double* cst, const float* part, int nslots, int64_t stride, int64_t M, hipStream_t s, const float* init = nullptr,
                       int init_mod = 0);
void launch_fill_zero(float* p, int64_t n, hipStream_t s);     // a kernel, so that captured launch sequences hold no memset node
// pk2[b][c] = (mu, nu with lambda in its sign bit: negative = 1), float2; columns n..ld-1 zero.
void launch_pack_relax2(const float* lambda, const float* mu, const float* nu, int batch, int n, int ld, float* pk2,
                        hipStream_t s);
// pk[side][b][c] = (0, 0, bound taken by C >= 0, bound taken by C < 0) for the concretisation.
void launch_pack_bounds(const float* lo, const float* hi, int batch, int n, int ld, float* pk, hipStream_t s);
// out[b, r] = float(cst[m] + sum over slots of part[slot][m]), m = (side*batch + b)*R + r.
// launch_finalize_bounds (both sides, R = n) and launch_relax_params_pack of the ReLU layer above in one launch.
void launch_finalize_relax_pack(const double* cst, const float* part, int nslots, int64_t part_stride, float* out_l, float* out_u,
                                float* lambda, float* mu, float* nu, float* rl, float* ru, const float* bias, int batch, int n, int ld,
                                float* pk, float* pk2, hipStream_t s);
// launch_finalize_bounds and launch_split_final of the merged last pass in one launch; false (nothing launched) when a
// group has more than 64 rows.
bool launch_finalize_split_final(const double* cst, const float* part, int nslots, int64_t part_stride, int batch, int nK, int Rs, float* l,
                                 float* u, float* margin, int32_t* verdict, hipStream_t s);
void launch_finalize_bounds(const double* cst, const float* part, int nslots, int64_t part_stride, int nsides, int batch,
                            int R, float* out_l, float* out_u, hipStream_t s);

// Margin rows of the robustness property: for input b and q-th other class o,
// row = W[label_b] - W[o], constant = bias[label_b] - bias[o].
void launch_margin_rows(const float* W, int ldw, const float* bias, const int32_t* label, int batch,
                        int nK, int n, float* C, int ldc, double* cst, hipStream_t s);

// Output-layer rows and margin rows stacked in one pass (2*nK - 1 rows per (side, input), held in groups of
// Rs >= 2*nK - 1 rows whose tail is zero; Rs = 0 means no padding); and the kernel that splits that pass's bounds
// ([batch][Rs] per side) into l,u of the output layer, margins and verdicts.
void launch_final_rows(const float* W, int ldw, const float* bias, const int32_t* label, int batch, int nK, int n,
                       float* C, int ldc, double* cst, hipStream_t s, int Rs = 0);
void launch_split_final(const float* tl, const float* tu, int batch, int nK, float* l, float* u, float* margin,
                        int32_t* verdict, hipStream_t s, int Rs = 0);

// verdict[b] = all margins of input b > 0.
void launch_verdict(const float* margin, int batch, int nq, int32_t* verdict, hipStream_t s);

// dst[b, perm(i)] = src[b, i] element permutation between (C,H,W) and (H,W,C) neuron orders.
void launch_chw_to_hwc(const float* src, float* dst, int batch, int C, int H, int W, hipStream_t s);
void launch_hwc_to_chw(const float* src, float* dst, int batch, int C, int H, int W, hipStream_t s);

}  // namespace dpc
