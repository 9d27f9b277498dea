/*
 * libftp - fused tile partitioning (FTP) of the feature-map dominated early layers of a CNN:
 * forward inference and back-propagation of K x K convolutions (K = 1, 3, 5, 7, stride 1 or 2; leaky ReLU folded
 * in; the 3x3 / 1x1 stride-1 layers of the paper's networks take the matrix-core kernels) and 2x2 max-pools, with feature and delta maps cut into an N x M grid of tiles, matching tiles of
 * consecutive layers fused into independent execution stacks, layers combined into groups that
 * exchange boundary (halo) data only at the group input, and per-stack partial filter
 * gradients summed once per batch (Sec. 3, Sec. 4.1, Sec. 4.2 of the paper).
 *
 * Plain C ABI.  Every pointer named "device" is a device (HBM) address on the current HIP
 * device; everything else is host memory.  The library owns only the plan (host memory).
 * It allocates no device memory: the caller provides all device buffers (sizes from
 * ftp_plan_sizes) and the stream.  The three device calls are asynchronous on `stream`.
 *
 * Numbering: boundary l (0..L) is the input of primitive layer l; boundary L is the output of
 * the network.  A group (s, e) covers primitive layers s..e-1 (Sec. 4.2).  Tile (ti, tj) has
 * row index ti in [0, N) and column index tj in [0, M); its stack index is ti*M + tj.
 * Rectangles are inclusive (x1, y1, x2, y2), x = column, y = row (Sec. 4.2).
 *
 * Layouts: maps NCHW contiguous; filters OIHW contiguous; element type per ftp_dtype
 * (FTP_BF16: 16-bit bfloat storage, fp32 accumulation; partial and reduced gradients are fp32
 * in both cases).  Parameter vector: concatenation over the convolution layers in layer order
 * of the filter (Cout*Cin*K*K) followed, if the layer has a bias, by the bias (Cout).
 *
 * A network without convolutions has no parameters (n_params = 0): the gradient pointers may then be null and the
 * gradient sum and the filter update do nothing.
 *
 * All functions return 0 on success or a negative ftp_status; nothing throws or aborts.
 *
 * A plan carries mutable host state (the event pool of the per-kernel timing, the second stream of the two-stream
 * backward pass): use one plan from one host thread at a time.  Different plans are independent.
 */
#ifndef FTP_H_
#define FTP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ftp_plan_s ftp_plan_t;

typedef enum { FTP_CONV = 0, FTP_MAXPOOL = 1 } ftp_layer_kind;
typedef enum { FTP_F32 = 0, FTP_BF16 = 1 } ftp_dtype;
typedef enum { FTP_RECT_OWN = 0, FTP_RECT_FWD = 1, FTP_RECT_BWD = 2 } ftp_rect_kind;

typedef enum {
    FTP_OK = 0,
    FTP_EINVAL = -1,        /* null pointer, non-positive size, index out of range            */
    FTP_EUNSUPPORTED = -2,  /* conv with stride not 1 or 2, K not in {1,3,5,7}, pad != K/2, pool != 2x2/2 */
    FTP_EGRID = -3,         /* a tile would own no pixel, a map too small for its pool, grid > 16 */
    FTP_EGROUPS = -4,       /* group ends not strictly increasing or not ending at n_layers    */
    FTP_ENOMEM = -5,        /* host allocation failed                                          */
    FTP_EHIP = -6,          /* a HIP call failed; see ftp_last_hip_error                       */
    FTP_ECHANNELS = -7,     /* cin of a layer does not match cout of the previous one          */
    FTP_ETOOLARGE = -8      /* the plan's workspace exceeds FTP_STATIC_WORKSPACE_BYTES (ftp_forward_static) */
} ftp_status;

/* One primitive layer (Sec. 4.2: kernel K_l x K_l, stride S_l).  FTP_CONV: K x K convolution, stride 1 or 2, zero
 * padding K/2 (an H-long map gives floor((H - 1)/S) + 1 positions), followed by leaky ReLU with `leaky_slope`
 * (Y = Z if Z > 0 else slope*Z; slope 1 gives a linear layer).
 * FTP_MAXPOOL: 2x2 window, stride 2, no padding (k = 2, stride = 2, pad = 0, cin == cout); on an odd map the last
 * row / column is left out (floor(H/2) positions) and receives a zero delta. */
typedef struct {
    int32_t kind, k, stride, pad, cin, cout;
    float leaky_slope;
    int32_t has_bias;
} ftp_layer;

/* Builds the partition plan (Sec. 4.2): map sizes, and per group and tile the owned rectangle
 * (equal split of the group's output map, projected back through the strides; the row / column a pool drops
 * from an odd map goes to the last tile), the forward
 * rectangles of Eq. (1) walked from e to s (what a stack computes and keeps), and the backward
 * (delta) rectangles of Eq. (2) walked from s to e; all clamped to the map.
 * Host only, integer only; touches no GPU.
 *   layers[n_layers]         primitive layers, in order
 *   batch, in_c, in_h, in_w  shape of the input map x
 *   grid_rows N, grid_cols M tile grid (1..16 each)
 *   group_ends[n_groups]     end boundary e of each group, strictly increasing, last == n_layers
 *   out_plan                 receives the plan; release with ftp_plan_destroy */
int ftp_plan(const ftp_layer* layers, int32_t n_layers,
             int32_t batch, int32_t in_c, int32_t in_h, int32_t in_w,
             int32_t grid_rows, int32_t grid_cols,
             const int32_t* group_ends, int32_t n_groups,
             ftp_dtype dtype, ftp_plan_t** out_plan);

void ftp_plan_destroy(ftp_plan_t* plan);

/* Rectangle of `kind` of tile (ti, tj) at `boundary` (s <= boundary <= e) of group `group`. */
int ftp_plan_rect(const ftp_plan_t* plan, int32_t group, int32_t boundary, int32_t ti, int32_t tj,
                  ftp_rect_kind kind, int32_t out_x1y1x2y2[4]);

/* (C, H, W) of the map at `boundary` (0..L). */
int ftp_plan_map_shape(const ftp_plan_t* plan, int32_t boundary, int32_t out_chw[3]);

/* Buffer sizes in bytes (any output pointer may be null):
 *   workspace_bytes      device scratch shared by ftp_forward and ftp_backward
 *   wgrad_partial_bytes  N*M*n_params*4
 *   n_params             length of the parameter vector
 *   per_stack_split[4]   what the largest stack has to hold: feature maps kept for back-propagation (recomputed
 *                        halo included), the delta maps alive at a time, filters + its own partial gradient set,
 *                        recorded decisions (pool winners, activation signs)  (the memory breakdown of Sec. 5.2) */
int ftp_plan_sizes(const ftp_plan_t* plan, size_t* workspace_bytes, size_t* wgrad_partial_bytes,
                   size_t* n_params, size_t per_stack_split[4]);

/* Work the plan implies, per batch (any pointer may be null):
 *   useful_macs    multiply-accumulates of the untiled network, forward + delta + filter gradient
 *   executed_macs  the same over the rectangles the stacks really evaluate (halo recompute included)
 *   halo_bytes[2]  bytes read outside the own tile at group boundaries, forward / backward */
int ftp_plan_work(const ftp_plan_t* plan, double* useful_macs, double* executed_macs, double halo_bytes[2]);

/* Where the plan keeps the map of `boundary` (for inspection and tests).  out[8] =
 *   [0] location: 0 none, 1 caller's x, 2 caller's y, 3 caller's dy, 4 caller's dx, 5 workspace
 *   [1] byte offset inside the workspace (location 5)
 *   [2] 1 if the buffer is a set of per-stack slots, 0 if it is one whole NCHW map
 *   [3] slot width, [4] slot height (whole map: W, H), [5] channels
 *   [6] rectangle kind whose top-left corner is the origin of each stack's slot (per-stack only)
 *   [7] group whose rectangles apply (per-stack only)
 * A per-stack buffer is laid out [stack][image][channel][slot height][slot width]; a stack's
 * rectangle occupies the top-left part of its slot.  Activations and deltas have the plan's type.
 * FTP_BUF_DELTA holds dLoss/dZ: where the boundary is the output of a convolution (with or without its
 * fused pool) the delta is dLoss/dY times the leaky-ReLU derivative there (Sec. 4.1, delta gradients);
 * for boundary L that is a scaled copy of the caller's dy kept in the workspace.
 * FTP_BUF_MASK (boundaries produced by a pool, fused or not) is the decision code of the forward
 * pass, one byte per element of a whole map, written by the owning stack: bit 0 = activation > 0,
 * bits 1-2 = index 2*dy+dx of the first maximum of the 2x2 window; back-propagation reads the
 * winners from it.  FTP_BUF_SIGN (outputs of convolutions, with or without fused pool) holds the
 * activation signs packed for back-propagation: whole map of 32-bit words [image][ceil(C/32)][H][W],
 * bit c%32 of word c/32 = activation of channel c > 0; out[5] is the number of words per pixel. */
typedef enum { FTP_BUF_ACT = 0, FTP_BUF_MASK = 1, FTP_BUF_DELTA = 2, FTP_BUF_SIGN = 3 } ftp_buf_kind;
int ftp_plan_buffer(const ftp_plan_t* plan, int32_t boundary, ftp_buf_kind which, int64_t out[8]);

/* Forward pass of all groups (Sec. 4.1 forward, Sec. 4.2 fusing and grouping).
 *   x        device, [batch][in_c][in_h][in_w]
 *   weights  host array of n_layers device pointers (filters, OIHW); entries of pool layers ignored
 *   biases   host array of n_layers device pointers, or null if no layer has a bias
 *   workspace device, workspace_bytes; keeps what ftp_backward needs
 *   y        device, output map [batch][C_L][H_L][W_L] */
int ftp_forward(const ftp_plan_t* plan, const void* x, const void* const* weights,
                const void* const* biases, void* workspace, void* y, void* stream);

/* ftp_forward for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops (forward inference), harnesses that forbid hipMalloc.  Same kernels, same launch order
 * and bit-identical y as ftp_forward, but the workspace is a fixed array of FTP_STATIC_WORKSPACE_BYTES that lives in
 * the library's device image (every GPU the library runs on holds its own copy until the process ends).  The call
 * allocates nothing, on the device or through any library.  Plans whose ftp_plan_sizes workspace_bytes exceed the
 * limit are rejected with FTP_ETOOLARGE before anything is launched.  x, weights, biases, y, stream as for
 * ftp_forward, on the current device.  The array keeps the previous call's contents (the forward pass needs
 * nothing cleared) and is shared by every call on that GPU: calls that overlap on one GPU (two streams, two threads)
 * race and must be serialised by the caller; ftp_backward cannot follow (it needs the caller's own workspace).
 * The first call on a device looks the array's address up (hipGetSymbolAddress); make that call outside a capture. */
#define FTP_STATIC_WORKSPACE_BYTES (64u * 1024u * 1024u)
int ftp_forward_static(const ftp_plan_t* plan, const void* x, const void* const* weights,
                       const void* const* biases, void* y, void* stream);

/* Back-propagation of all groups in reverse (Sec. 4.1 delta and filter gradients).
 *   dy        device, dLoss/dy, shape of y
 *   x         device, the input of the preceding ftp_forward on the same workspace
 *   dx        device, receives dLoss/dx, shape of x
 *   wgrad_partials device, fp32 [N*M][n_params]: one partial parameter gradient per stack, summed
 *             over the batch and over the output pixels the stack owns; overwritten, not accumulated */
int ftp_backward(const ftp_plan_t* plan, const void* dy, const void* x,
                 const void* const* weights, void* workspace, void* dx,
                 float* wgrad_partials, void* stream);

/* wgrad[p] = sum over the N*M stacks of wgrad_partials[stack][p] (Sec. 4.1: the partial sums of
 * the tiles simply add up; done once per batch for all filters of all layers).  Fixed balanced
 * pairwise order over the stack index, so results are bitwise reproducible.
 *   wgrad_partials device fp32 [N*M][n_params];  wgrad device fp32 [n_params] */
int ftp_reduce_wgrad(const ftp_plan_t* plan, const float* wgrad_partials, float* wgrad, void* stream);

/* Gradient sum fused with the filter update that closes a training cycle (Sec. 4.1: the final
 * gradient "can then be used to update" the filters, once per batch for all layers).  The paper
 * names no optimiser; this is the plain gradient-descent step
 *   W_l[i] <- W_l[i] - lr * sum over stacks of wgrad_partials[stack][offset_l + i]
 * (biases likewise), with the same summation order as ftp_reduce_wgrad.  Arithmetic in fp32; with
 * FTP_BF16 the updated value is rounded to the storage type.
 *   weights, biases  host arrays of n_layers device pointers as for ftp_forward, updated in place
 *                    (biases may be null if no layer has one)
 *   wgrad            device fp32 [n_params] or null: also receives the summed gradient */
int ftp_sgd_step(const ftp_plan_t* plan, const float* wgrad_partials, void* const* weights, void* const* biases,
                 float lr, float* wgrad, void* stream);

/* Backward pass on two streams (Sec. 4.1: the delta back-propagation and the filter gradients of a layer both start
 * from the same delta map and do not depend on each other).  When enabled, ftp_backward runs each unit's filter
 * gradient on a second HIP stream of its own (default priority; the stream and the events of one pass are host
 * objects created by this call and owned by the plan, so that ftp_backward creates nothing and can be captured into a
 * HIP graph with the switch on; if no device is usable yet, they are created by the first ftp_backward instead) beside the unit's delta back-propagation on the caller's stream, ordered with events so that no kernel
 * overwrites a map another one still reads; before ftp_backward returns, the caller's stream has been made to wait for
 * the second one, so the caller sees one stream as before.  Results are bit-identical either way.  Off by default
 * (on if the environment variable FTP_OVERLAP is 1 when the plan is created).  Kernels that run side by side share the
 * GPU, so the per-kernel records of ftp_profile then show longer launches while the whole pass gets shorter. */
int ftp_set_overlap(ftp_plan_t* plan, int32_t enable);

/* Per-kernel timing for benchmarks.  While enabled, every kernel launch of the three passes is
 * bracketed by two HIP events on the caller's stream (host objects, created on first use and
 * owned by the plan).  ftp_profile(plan, 1) clears earlier records and starts collecting,
 * ftp_profile(plan, 0) stops.  ftp_profile_read waits for the recorded events and returns one
 * record per (pass, layer): number of launches, their summed duration, and the algorithmic
 * work of one launch - the FLOPs and HBM bytes of the untiled layer (each map read or written
 * once, recomputed halos not credited) - and, beside it, the FLOPs the launch really executed.  `count` receives the number of records available;
 * at most `capacity` are written to `out` (host). */
typedef enum {
    FTP_PASS_CONV_FWD = 0, FTP_PASS_CONV_BWD_DATA = 1, FTP_PASS_WGRAD = 2, FTP_PASS_REDUCE = 3,
    FTP_PASS_POOL_FWD = 4, FTP_PASS_POOL_BWD = 5,
    FTP_PASS_SCALE_DY = 6,         /* dy times the last activation's derivative; layer = last convolution */
    FTP_PASS_UPDATE = 7,           /* ftp_sgd_step; layer = the convolution updated */
    FTP_PASS_WGRAD_SUM = 8         /* sum of the batch shares of a layer's per-stack filter gradient (inside ftp_backward) */
} ftp_pass;
typedef struct {
    int32_t pass, layer, launches, reserved;   /* layer = primitive layer index, -1 for the reduction */
    double total_ms, flops_per_launch, bytes_per_launch;
    char kernel[96];                           /* name of the kernel the launches ran */
    double executed_flops_per_launch;          /* the same FLOPs over the rectangles the stacks really evaluate: forward
                                                  and delta passes recompute the halo inside a group (Sec. 4.2), the
                                                  filter gradient runs over owned pixels only (equal to flops_per_launch) */
} ftp_kernel_time;
int ftp_profile(ftp_plan_t* plan, int32_t enable);
int ftp_profile_read(ftp_plan_t* plan, ftp_kernel_time* out, int32_t capacity, int32_t* count);

const char* ftp_strerror(int code);

/* hipError_t value of the last failed HIP call on this thread (0 if none). */
int ftp_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FTP_H_ */
