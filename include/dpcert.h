/*
 * dpcert -- DeepPoly-style symbolic bound propagation on one AMD MI355X (gfx950).
 *
 * C ABI.  Every function returns a dpc_status (0 = OK) and never throws; the
 * text of the last error on the calling thread is available from
 * dpc_last_error().  Unless a parameter says "device", pointers may be host or
 * device memory: the library copies through hipMemcpy's default (address
 * inferring) kind and never keeps a caller pointer after the call returns.
 *
 * Problem statement (paper, Section 2): a property is a pair (phi, psi); the
 * certifier attaches an abstract shape (l, u, L, U) to every neuron -- concrete
 * bounds l <= eta <= u and polyhedral bounds L <= eta <= U, each polyhedral
 * expression being c0 + sum_i c_i * eta_i (Section 2.1) -- starting from phi on
 * the input layer, propagates it with abstract transformers, and compares the
 * output constraints with psi: the result is "verified" or "unknown".
 * Here phi is an axis-aligned box [lo, hi] per input (an L-infinity ball) and
 * psi is "logit[label] is larger than every other logit".
 *
 * Method (paper, Appendix C, DeepPoly specification):
 *   Affine / convolution neuron:  L = U = prev.dot(w) + b;  l = backsubs_lower(L),
 *     u = backsubs_upper(U): traverse the network backwards, replacing every
 *     term c*eta by c*L_eta or c*U_eta according to the sign of c, layer after
 *     layer until only input neurons remain, then replace c*eta by c*l_eta or
 *     c*u_eta by sign and sum (Sections 2.1, 2.2; Appendix C).
 *   ReLU neuron over predecessor p with bounds (l, u):
 *     l' = max(l,0), u' = max(u,0);  L = (l + u >= 0) ? p : 0;
 *     U = l >= 0 ? p : (u <= 0 ? 0 : u/(u-l) * p - u*l/(u-l)).
 *   The library reports L of a ReLU neuron as lambda*p and U as mu*p + nu.
 *
 * Layer indices: 0 is the input layer, i >= 1 is the i-th dpc_network_add_* call.
 * Neurons of a convolution layer are numbered (channel, row, column) row-major,
 * on both sides of this interface (weights of a following affine layer use the
 * same order); zero padding.
 */
#ifndef DPCERT_H
#define DPCERT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t dpc_status;
enum {
    DPC_OK = 0,
    DPC_EINVAL = 1,        /* null pointer, bad dimension, size chain mismatch, lo > hi, label out of range, non-finite value */
    DPC_EUNSUPPORTED = 2,  /* ReLU as first layer, two ReLUs in a row, ReLU after the last affine layer */
    DPC_ENOMEM = 3,        /* host or device allocation failed */
    DPC_EHIP = 4,          /* a HIP call failed; dpc_last_error() holds its message */
    DPC_ESTATE = 5         /* wrong call order (certify before finalize, add after finalize, ...) */
};

typedef struct dpc_network dpc_network;   /* opaque; owned by the library until dpc_network_destroy */
typedef struct dpc_result dpc_result;     /* opaque; owned by the library until dpc_result_destroy  */

/* ---- network description (host side; Section 2: the DNN is the graph the certifier walks) ---- */

dpc_status dpc_network_create(dpc_network** out);

/* Fully-connected layer y = W x + b.  W: [out_dim, in_dim] row-major, b: [out_dim];
 * both are copied.  in_dim must equal the previous layer's size. */
dpc_status dpc_network_add_affine(dpc_network* net, int32_t out_dim, int32_t in_dim,
                                  const float* W, const float* b);

/* 2-D convolution (cross-correlation, zero padding) on a (Ci, H, W) input.
 * K: [Co, Ci, kh, kw] row-major, b: [Co]; copied.  Ci*H*W must equal the
 * previous layer's size.  Output (Co, Ho, Wo), Ho = (H + 2*pad - kh)/stride + 1.
 * The layer is an affine layer whose weight matrix is the expanded kernel
 * (Section 3.3); the library never materialises that matrix. */
dpc_status dpc_network_add_conv2d(dpc_network* net, int32_t Ci, int32_t H, int32_t W,
                                  int32_t Co, int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                  const float* K, const float* b);

/* ReLU over the previous layer (element-wise). */
dpc_status dpc_network_add_relu(dpc_network* net);

/* Add layer of a residual network: neuron i = neuron i of the previous layer + neuron i of layer
 * `from_layer` (0 = the network input, k = the k-th layer added; it must lie below the previous
 * layer and have the same size and, for convolutional layers, the same shape).  The paper's
 * specification language names two predecessors (prev0, prev1) but prints no Add transformer; the
 * library reads it as the Affine transformer with unit weights over both: L = U = prev0 + prev1,
 * l, u by back-substitution.  A polyhedral expression that crosses the layer then has terms on two
 * layers at once: two blocks of one coefficient tensor (Section 5.1), which are summed when the
 * traversal brings them onto the same layer (Section 5.2, overlapping blocks are merged); the
 * deepest layer is always replaced first (Section 4.2).  The previous layer may be of any kind: above a
 * fully-connected or convolution layer the traversal starts from that layer's rows, above a ReLU or another
 * Add layer from coefficient 1 on each operand (two Diagonal blocks, Section 3.3).  A depth-limited traversal that stops while a
 * block still waits on a skip connection concretises the expression over both layers it holds.
 * ReuseCert is specified for chain networks: dpc_certify returns DPC_EUNSUPPORTED. */
dpc_status dpc_network_add_skip(dpc_network* net, int32_t from_layer);

/* Validate the chain, upload weights to HIP device `device` in the layouts the
 * kernels use.  After this call no layer can be added.  Synchronous. */
dpc_status dpc_network_finalize(dpc_network* net, int32_t device);

/* Frees host and device memory of the network (results must be destroyed first). */
dpc_status dpc_network_destroy(dpc_network* net);

/* ---- certification ---- */

typedef struct {
    int32_t struct_size;        /* = sizeof(dpc_options); rejects mismatching callers */
    int32_t max_backsub_depth;  /* -1: traverse to the input (DeepPoly).  p >= 0: at most p traverse
                                   iterations (each replaces one layer's neurons, ReLU layers
                                   included), then concretise against the stored l,u of the layer
                                   reached -- the DeepPoly_p family of Section 6.2; 0 = IBP */
    int32_t keep_symbolic;      /* which neurons' polyhedral bounds L, U (Section 2.1: the symbolic half of the abstract shape),
                                   back-substituted to the input layer, stay available after the call: 0 none; 1 the
                                   last layer's and the property rows' (needs final_backsub_depth = -1); 2 those of
                                   every affine, convolution and Add layer (needs max_backsub_depth = -1 too; every
                                   traversal then runs step by step: 2*batch*n_layer*n0 floats are kept per layer) */
    int32_t fuse;               /* 1 (default): the ReLU step / concretisation that follows a
                                   contraction runs in that contraction's epilogue where supported;
                                   0: every step is its own kernel */
    int32_t profile;            /* 1: time every kernel class with HIP events (see dpc_result_profile) */
    int32_t use_graph;          /* 1 (default): when a result object is reused on a non-null stream, the call's kernel
                                   sequence is captured into a HIP graph once and replayed (launch-bound small networks);
                                   0: always launch kernel by kernel */
    int32_t certifier;          /* DPC_DEEPPOLY (0, default) or DPC_REUSECERT (1): every affine layer keeps its bounds
                                   already back-substituted to the input and later layers reuse them, one replacement
                                   step per layer (Appendix C, ReuseCert; Section 6.1).  Chain networks with affine or
                                   convolution layers and ReLU layers alternating (the step through a convolution layer
                                   contracts its split kernel matrix with the stored rows its window touches, held dense
                                   over the input); needs max_backsub_depth = -1 and
                                   keep_symbolic = 0.  dpc_result_concrete then returns, for an affine layer, the
                                   concretisation of its stored bounds (the values the next ReLU transformer uses) */
                                /* DPC_SKIPPOLY (2): DeepPoly whose ReLU neurons carry their polyhedral bounds over the neurons two
                                   layers back (Appendix C, SkipPoly; Section 6.1): L = lambda * (w . prev2 + b), U = mu * (w . prev2 + b)
                                   + nu with (w, b) the row of the layer under the ReLU neuron, so a traverse iteration replaces a
                                   ReLU layer and the layer under it at once (half as many iterations, same bounds).  That is
                                   the step the fused kernels execute; the certifier selects it and makes the ReLU neurons'
                                   shape available from dpc_result_relu_symbolic.  Chain networks, full traversals only */
    int32_t final_backsub_depth; /* traversal limit of the LAST layer and of the property (margin) rows: DPC_SAME_DEPTH
                                   (-2, default) = max_backsub_depth; -1 = to the input; p >= 0 as above.
                                   max_backsub_depth = 0 with final_backsub_depth = -1 is CROWN-IBP (Appendix C): interval
                                   bounds for every hidden layer, full back-substitution for the output constraints */
    void*   stream;             /* hipStream_t all work is enqueued on (NULL = the null stream) */
} dpc_options;
enum { DPC_SAME_DEPTH = -2 };
enum { DPC_DEEPPOLY = 0, DPC_REUSECERT = 1, DPC_SKIPPOLY = 2 };

/* Fills `opt` with the defaults (full traversal, nothing kept, fused, no profile, graph replay on, null stream). */
dpc_status dpc_options_default(dpc_options* opt);

/* Runs the certifier on `batch` boxes: the forward flow of Appendix C (DeepPoly) -- layers in order, each affine /
 * convolution / Add layer bounded by one backward traversal of its neurons' expressions (Section 2.2, traverse;
 * Sections 3.2 and 4.3 for the tensor form of one iteration), each ReLU layer by its transformer -- then the
 * property check of Section 2 (psi against the output layer's constraints).
 *   lo, hi : [batch, n0] float32, lo <= hi element-wise (host or device).
 *   label  : [batch] int32 target class in [0, nK), or NULL for bounds only.
 *   *result: NULL -> a new result is allocated; a result returned by an earlier
 *            call on the same network with the same batch and keep_symbolic ->
 *            it is reused and no device memory is allocated.
 * Work is enqueued on opt->stream; the call returns after the stream has been
 * synchronised, so results are ready.  The boxes and labels are validated on the
 * device while the certifier runs (lo > hi, a non-finite bound or a label out of
 * range -> DPC_EINVAL, found when the stream is synchronised; a label out of range is
 * clamped inside the kernels so that nothing is read out of bounds); after such an
 * error the contents of a reused result are unspecified and no new result is returned.  Calls on one network must not overlap
 * (the network owns the coefficient workspace). */
dpc_status dpc_certify(dpc_network* net, int32_t batch, const float* lo, const float* hi,
                       const int32_t* label, const dpc_options* opt, dpc_result** result);

/* dpc_certify for callers that cannot allocate device memory: code that runs under a HIP graph capture or inside a
 * region where hipMalloc is forbidden, tight serving loops, harnesses that track every allocation.  The call makes
 * no hipMalloc / hipFree / hipHostMalloc and creates no result object: its whole workspace (coefficient rows, row
 * constants, packed parameters, every layer's bounds) is carved out of ONE array of 64 MiB that the library holds
 * in static device memory on each device it runs on, from load time until the process ends.
 *   lo, hi, label : as for dpc_certify, but DEVICE memory of the network's device (DPC_EINVAL otherwise).
 *   out_l, out_u  : [batch, nK] float32 device, bounds of the last layer (either may be NULL).
 *   margin_lb     : [batch, nK-1] float32 device, verdict: [batch] int32 device (may be NULL; need a label).
 *   opt           : certifier DPC_DEEPPOLY with any depth limits; keep_symbolic must be 0; profile and use_graph
 *                   are ignored (DPC_EUNSUPPORTED for ReuseCert, kept symbolic bounds, the split-precision tuning).
 * A problem whose workspace exceeds the 64 MiB is rejected with DPC_EINVAL before anything is launched (the
 * message says so); dpc_certify takes it.  Results equal dpc_certify's bit for bit (same kernels, same order).
 * Every call on a device uses that device's one array, which keeps the previous call's contents (what has to
 * start at zero is cleared by a kernel of the call): calls that overlap on one device race, also on different
 * networks.  Returns after the stream has been synchronised. */
dpc_status dpc_certify_static(dpc_network* net, int32_t batch, const float* lo, const float* hi, const int32_t* label,
                              const dpc_options* opt, float* out_l, float* out_u, float* margin_lb, int32_t* verdict);

/* Concrete bounds l, u of the abstract shape (Section 2.1; Appendix C, DeepPoly shape) of every neuron of `layer` (0 = the box itself):
 * [batch, n_layer] float32 each, caller-allocated (host or device); either may be NULL. */
dpc_status dpc_result_concrete(const dpc_result* res, int32_t layer, float* l, float* u);

/* Polyhedral bounds of the neurons of ReLU layer `relu_layer` over their
 * predecessors: L = lambda*p, U = mu*p + nu.  [batch, n] float32 each; any may be NULL. */
dpc_status dpc_result_relaxation(const dpc_result* res, int32_t relu_layer,
                                 float* lambda, float* mu, float* nu);

/* Polyhedral bounds L (side 0) and U (side 1) of the neurons of an affine, convolution or Add layer, in the form the
 * traversal leaves them in when only input neurons remain (Section 2.2; Appendix C, backsubs_lower / backsubs_upper
 * before simplify_* is mapped over them):  L_r(x) = cst[b,r] + sum_i coeff[b,r,i] * x_i <= neuron r <= U_r(x) on the box.
 * coeff [batch, n_layer, n0], cst [batch, n_layer], caller-allocated (host or device); either may be NULL.  Rows and
 * columns are in the interface's neuron order ((C,H,W) for spatial layers).  Needs keep_symbolic = 1 (last layer) or 2
 * (any such layer); DPC_ESTATE otherwise; ReLU layers: DPC_EINVAL (their L, U over the predecessor are lambda, mu, nu). */
dpc_status dpc_result_symbolic(const dpc_result* res, int32_t layer, int32_t side,
                               float* coeff, float* cst);

/* SkipPoly shape of the neurons of ReLU layer `relu_layer` (Appendix C, SkipPoly: relu_n and compute_upper applied to
 * the L, U of the neuron underneath): their polyhedral bounds over the layer two below, L (side 0) = lambda * (w . prev2
 * + b), U (side 1) = mu * (w . prev2 + b) + nu.  coeff [batch, n, n_prev2], cst [batch, n] (host or device; either may be
 * NULL), neuron orders as in dpc_result_symbolic; the layer under the ReLU layer must be fully-connected or a convolution
 * (its expanded kernel rows are written out).  Needs certifier = DPC_SKIPPOLY at certify time (DPC_ESTATE otherwise). */
dpc_status dpc_result_relu_symbolic(const dpc_result* res, int32_t relu_layer, int32_t side, float* coeff, float* cst);

/* The same for the property rows (keep_symbolic >= 1 and labels): the lower polyhedral bound, over the input, of
 * logit[label] - logit[o] for o != label in ascending o; coeff [batch, nK-1, n0], cst [batch, nK-1].  Its minimum over
 * the box is margin_lb of dpc_result_verdict. */
dpc_status dpc_result_margin_symbolic(const dpc_result* res, float* coeff, float* cst);

/* Outcome of the property check (Section 2: certified, or unknown when the property does not hold or the analysis is too
 * imprecise).  verdict [batch]: 1 = verified, 0 = unknown.  margin_lb [batch, nK-1] (may be
 * NULL): lower bound of logit[label] - logit[o] for o != label in ascending o.
 * Verified iff every margin lower bound is > 0.  Needs a label at certify time. */
dpc_status dpc_result_verdict(const dpc_result* res, int32_t* verdict, float* margin_lb);

/* Per-kernel-class timing of the certify call that produced `res` (opt->profile = 1).
 * Times are sums of HIP-event intervals on the call's stream, in milliseconds;
 * flop / byte counts are the algorithmic ones of the launches made. */
typedef struct {
    int32_t struct_size;
    int32_t contract_launches, relax_launches, concretise_launches, other_launches;
    double  contract_ms, relax_ms, concretise_ms, other_ms, total_ms;
    double  contract_flop;       /* 2*M*K*N per contraction (conv: compressed-core count) */
    double  relax_bytes;         /* 8 B per coefficient (first step of a pass: 4 B) */
    double  concretise_bytes;    /* 4 B per coefficient */
    /* whole traversals run as one LDS-resident kernel (not included in the contract_* fields) */
    double  chain_ms;
    double  chain_flop;          /* sum of 2*M*K*N over the layers each launch crosses */
    int32_t chain_launches;
    int32_t reserved;
} dpc_profile;
dpc_status dpc_result_profile(const dpc_result* res, dpc_profile* out);

/* Frees the result's device and host memory (the abstract shapes of Section 2.1 it holds). */
dpc_status dpc_result_destroy(dpc_result* res);

/* ---- the three hot kernels on caller-owned DEVICE buffers (unit tests, roofline runs) ---- */

/* Affine contraction of a traverse iteration (Matmul rewrite, Section 4.3):
 *   Cout[m, 0:N] = sum_k A[m, k] * W[k, 0:N],  m < M, k < K.
 * A: [M, lda] device, W: [K, ldw] device, Cout: [M, ldc] device, all float32 row-major;
 * lda >= K, ldw >= N, ldc >= N.  Columns N..ldc-1 of Cout are written as zero.
 * Requirements (EINVAL otherwise): lda, ldw, ldc multiples of 4; buffers 16-byte aligned. */
dpc_status dpc_op_contract(const float* A, int64_t M, int32_t K, int32_t lda,
                           const float* W, int32_t N, int32_t ldw,
                           float* Cout, int32_t ldc, void* stream);

/* Sign-split ReLU step of a traverse iteration (replace_lower / replace_upper with the
 * Ternary and Clamp rewrites of Section 4.3) followed by the bias fold of the affine
 * layer below.  Rows are ordered [side][input][r]: m = (side*batch + b)*R + r, side 0 = lower.
 *   lower rows: C'[m,i] = max(C,0)*lambda[b,i] + min(C,0)*mu[b,i];  c' = c + sum_i min(C,0)*nu[b,i]
 *   upper rows: C'[m,i] = max(C,0)*mu[b,i] + min(C,0)*lambda[b,i];  c' = c + sum_i max(C,0)*nu[b,i]
 *   both      : c' += sum_i C'[m,i] * bias[i]
 * C: [nsides*batch*R, ldc] device float32, updated in place; cst: [nsides*batch*R] device float64,
 * updated in place; lambda, mu, nu: [batch, n] device; bias: [n] device.  If shared_src is not
 * NULL it is a [R, ld_src] matrix read instead of C for every (side, b) (the weight rows of the
 * layer being bounded, which carry no batch dimension before the first ReLU step). */
dpc_status dpc_op_relax_step(float* C, int32_t ldc, double* cst, int32_t nsides, int32_t batch, int32_t R,
                             int32_t n, const float* lambda, const float* mu, const float* nu,
                             const float* bias, const float* shared_src, int32_t ld_src, void* stream);

/* Concretisation (simplify_lower / simplify_upper, Appendix C) against the box:
 *   lower rows: out_l[b,r] = c + sum_i (C >= 0 ? C*lo[b,i] : C*hi[b,i])
 *   upper rows: out_u[b,r] = c + sum_i (C >= 0 ? C*hi[b,i] : C*lo[b,i])
 * Row order as in dpc_op_relax_step.  out_l, out_u: [batch, R] device float32
 * (out_u unused when nsides = 1). */
dpc_status dpc_op_concretise(const float* C, int32_t ldc, const double* cst, int32_t nsides, int32_t batch,
                             int32_t R, int32_t n, const float* lo, const float* hi,
                             float* out_l, float* out_u, void* stream);

/* Convolution contraction of a traverse iteration: coefficient rows over a convolution layer's
 * outputs times its Convolution block (Appendix B.3: dense block x convolution block is a
 * transposed convolution), never forming the expanded matrix.  Channel-last rows:
 *   in : [M][ih][iw][Co] device, rows ld_in floats apart;  out: [M][oh][ow][Ci] device, ld_out apart
 *   out[m,y,x,ci] = sum over (ky,kx,co) with y+off-ky = py*stride, x+off-kx = px*stride,
 *                   0 <= py < ih, 0 <= px < iw, of in[m,py,px,co] * K[co,ci,ky,kx]
 * K: [Co,Ci,kh,kw] HOST memory (uploaded for the call).  off = the layer's padding when the rows
 * cover the whole output map, 0 for patch rows.  Columns oh*ow*Ci..ld_out-1 of out are zeroed.
 * Synchronises the stream before returning. */
dpc_status dpc_op_conv_transpose(const float* in, int64_t M, int32_t ld_in, int32_t ih, int32_t iw,
                                 int32_t Co, int32_t Ci, int32_t kh, int32_t kw, int32_t stride, int32_t off,
                                 const float* K_host, float* out, int32_t ld_out, int32_t oh, int32_t ow,
                                 void* stream);

/* Tuning knob for experiments: key "contract_variant" selects the tile shape of the contraction
 * kernel (-1 = chosen from the problem shape, the default); key "conv_algo" = 1 forces the generic
 * gather kernel for convolution contractions (0 = MFMA / small-channel kernels where they apply);
 * key "chain" chooses when the traversal of a fully-connected layer's rows runs as one kernel with the
 * coefficient rows resident in LDS (-1 = by problem shape, the default; 0 = never; 1 = whenever the
 * layer widths fit) and "chain_rows" its row block for panels up to 512 columns (64, the default, or 32 with two
 * workgroups per compute unit); "conv_algo" = 2 sends few-input-channel layers to the plain-ALU kernel;
 * "conv_half_tiles" = 0 keeps 32 x 32 tiles in the matrix-unit convolution kernel also for layers with at most 16
 * input channels (1, the default, uses 16 x 16 tiles there);
 * "merge_final" = 0 bounds the output layer and the margins in two traversals instead
 * of one; "contract_remap", "rows_per_wave", "rows_stream", "stream_wgs_per_cu" select launch shapes of the contraction and
 * row kernels; "reuse_patch" = 0 keeps ReuseCert's stored bounds of convolution layers as rows over the whole input,
 * "reuse_window" = 0 gathers the rows a convolution layer reads before contracting them, "reuse_window_ck" (8..64)
 * and "reuse_window_tiles" (0 rows, 1 flat) select the chunk and tile shape of the implicit contraction.  Results do not depend on any of them beyond rounding order.
 * Split-precision experiment (the exception to that sentence): "contract_split" = 2 or 3 (default 0) runs
 * the contractions through fully-connected layers on the bf16 matrix units with both operands written as
 * sums of 2 or 3 bf16 terms and the 3 or 6 largest partial products accumulated in fp32 ("bf16x3": about
 * 16 significand bits per product, "bf16x6": about 24); layers whose size is not a multiple of 4 and all
 * convolutions stay on the fp32 kernels; the resident traversal kernel is not used.  "contract_split_wide"
 * (-1 by shape, 0, 1) selects its 128 x 256 tile. */
dpc_status dpc_tuning_set(const char* key, int32_t value);

/* The same knobs for one network: calls on `net` (and reads of its results) use `value` for `key` whatever the
 * process-wide value is; DPC_TUNING_DEFAULT as the value removes the override.  The process-wide values are read
 * atomically and the values in force for a call are fixed when it starts, so dpc_tuning_set on one thread does not
 * disturb a call running on another, and calls on different networks from different threads do not share knob
 * state.  (Calls on one network still must not overlap: they share its workspace.)  For callers that cannot
 * serialise process-wide settings: services that certify several networks from several threads.
 * DPC_EINVAL for an unknown key. */
#define DPC_TUNING_DEFAULT INT32_MIN
dpc_status dpc_network_tuning_set(dpc_network* net, const char* key, int32_t value);

/* Text of the last error raised on the calling thread ("" if none). */
const char* dpc_last_error(void);

/* Library version string. */
const char* dpc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DPCERT_H */
