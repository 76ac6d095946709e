/*
 * resist.h -- C ABI of the MI355X (gfx950) library for the data-parallel hot path of ResIST:
 * the random layer-wise split of a global ResNet into S sub-ResNets, one local SGD iteration
 * of one sub-ResNet, and the reassembly that averages blocks shared between sub-ResNets
 * (the paper's Algorithm 1: subResNets(), the inner update W_s <- W_s - eta dL/dW_s, aggregate()).
 *
 * Conventions common to every call
 *   - Return value: 0 (RESIST_OK) or a negative resist_status; resist_last_error() then holds a
 *     message.  No exception or abort crosses this boundary; arguments are validated before any
 *     kernel is launched.
 *   - "device" pointers are HIP device memory owned by the caller (16-byte aligned); the library
 *     allocates no device memory and returns without synchronising.  "host" pointers are ordinary
 *     memory.  Seen from the caller, everything a call enqueues is ordered on the stream it passes.
 *   - Process-wide state the library does keep: (a) per device, one second HIP stream (default
 *     priority, non-blocking) and a ring of 256 events, created at the first resist_local_step that
 *     uses them and kept until the process ends: the weight-gradient kernels of a step (and the few
 *     other kernels its dependent chain does not wait for: shortcut convolutions of the forward pass,
 *     the head's parameter gradients, the mean loss) run there, ordered against the caller's stream
 *     by those events (resist_set_overlap); (b) the
 *     resist_set_overlap and resist_set_bn_fusion modes; (c) the optional timing facility
 *     (resist_profile_*); (d) 32 MiB of static device memory per GPU behind
 *     resist_conv2d_wgrad_static (resist_ops.h).
 *   - Threads: host-only calls are reentrant.  Calls that enqueue work on the same device must not
 *     overlap in time from different host threads (the event ring is shared per device); different
 *     devices may be driven from different threads.
 *   - Same inputs give bit-identical outputs from run to run (no floating-point atomics).
 *   - Blocks of the global network are numbered 0..B-1 in network order; -1 names the stem and
 *     B the head (global pooling + fully connected layer).  Stem and head belong to every
 *     sub-ResNet (Sec. 2.2: initial and final layers are shared; Appendix B: the last layer is
 *     never dropped).
 *
 * Parameter buffers.  Every block (and the stem, and the head) owns ONE contiguous fp32 buffer:
 *     [ trainable tensors ... | BN running statistics ... ]
 *   trainable part, in order: conv1 W, bn1 gamma, bn1 beta, conv2 W, bn2 gamma, bn2 beta,
 *   [conv3 W, bn3 gamma, bn3 beta,] [downsample W, its gamma, its beta]; stem: conv W, gamma,
 *   beta; head: fc W [classes][C], fc bias.  Pre-activation kinds: bn1 gamma, beta, conv1 W, bn2
 *   gamma, beta, conv2 W, [bn3 gamma, beta, conv3 W,] [downsample W]; stem: conv W; head: bn
 *   gamma, beta, fc W, fc bias.  Then running mean, running var of each BN in the
 *   same order.  Each tensor starts at a multiple of 4 floats (zero padding after it if needed).
 *   Convolution weights are stored [K][R][S][C] (output channel, filter row, filter column, input
 *   channel; C fastest), i.e. element (k,c,r,s) of the logical [K,C,R,S] filter sits at
 *   ((k*R + r)*S + s)*C + c.  resist_block_layout() reports every tensor's offset and shape.
 *   Momentum and gradient buffers mirror the trainable part (the first n_trainable floats).
 *   Activations inside the library are NHWC; the input batch is passed as logical [N,C,H,W].
 */
#ifndef RESIST_H
#define RESIST_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RESIST_MAX_STAGES 4

typedef enum {
  RESIST_OK = 0,
  RESIST_EINVAL = -1,     /* bad argument value (NULL, negative size, S < 1, unknown kind ...)   */
  RESIST_ESHAPE = -2,     /* model description / block list inconsistent with what kernels need   */
  RESIST_EWORKSPACE = -3, /* workspace or output capacity too small                               */
  RESIST_EHIP = -4,       /* a HIP runtime call or kernel launch reported an error                */
  RESIST_EUNSUPPORTED = -5
} resist_status;

/* The GLOBAL ResNet (Sec. 2.1: sections of blocks of equal channel width).  Plain data. */
typedef struct {
  int32_t block_kind;    /* 0 basic: conv3x3-BN-ReLU-conv3x3-BN, +shortcut, ReLU
                            1 bottleneck: conv1x1-BN-ReLU-conv3x3-BN-ReLU-conv1x1(x4)-BN, +, ReLU
                            2, 3: the same two in pre-activation form (Sec. 2.1, Fig. 2):
                               BN-ReLU before every convolution, shortcut added without a ReLU;
                               the stem is the bare convolution (stem_kind 0 only), the head starts
                               with BN-ReLU, a shape-changing shortcut is conv1x1(stride) applied to
                               the block's first ReLU output, without BN                          */
  int32_t stem_kind;     /* 0: conv3x3 stride 1 pad 1, BN, ReLU
                            1: conv7x7 stride 2 pad 3, BN, ReLU, maxpool 3x3 stride 2 pad 1       */
  int32_t in_c, in_h, in_w;
  int32_t num_stages;                 /* 1..RESIST_MAX_STAGES                                    */
  int32_t width[RESIST_MAX_STAGES];   /* channel width per stage (multiple of 16)                */
  int32_t blocks[RESIST_MAX_STAGES];  /* residual blocks per stage (>= 1)                        */
  int32_t num_classes;
  int32_t compute_dtype; /* 0: fp32 MFMA.  1: bf16 MFMA operands, fp32 accumulate, fp32 masters  */
  float bn_eps;
  float bn_momentum;
} resist_model_desc;
/* The first block of stage i > 0 has stride 2 (on its 3x3 convolution); a first block whose input
 * and output shapes differ gets a conv1x1(stride)-BN shortcut; all other shortcuts are identity. */

typedef struct {
  int32_t kind;     /* 0 conv weight, 1 BN gamma, 2 BN beta, 3 BN running mean, 4 BN running var,
                       5 FC weight, 6 FC bias                                                    */
  int32_t layer;    /* 0 conv1 (or the stem conv / the FC), 1 conv2, 2 conv3, 3 downsample        */
  int64_t offset;   /* in floats from the start of the block buffer                              */
  int64_t count;    /* number of floats (without padding)                                        */
  int32_t dims[4];  /* conv: K,R,S,C;  vector: C,0,0,0;  FC weight: classes,C,0,0                */
} resist_tensor_info;

/* Number of residual blocks B of the global network.  host. */
int resist_num_blocks(const resist_model_desc *desc, int32_t *num_blocks);

/*
 * Random layer-wise split (Sec. 2.2; Sec. 2.6 "Subnetwork Depth"): the indices of the partitionable
 * blocks are permuted at random and dealt round-robin so that every sub-ResNet receives the same
 * number D = max(ceil(P/S), min(min_depth, P)) of them; sub s takes permuted positions
 * s, s+S, s+2S, ... (mod P), skipping forward over blocks it already holds, so blocks are shared
 * when S does not divide P or the depth floor asks for it.  Non-partitionable blocks go to every
 * sub-ResNet.  Random source: splitmix64 with state seed ^ (round * 0x9E3779B97F4A7C15),
 * Fisher-Yates from the top index down with j = next() mod (i+1).  Pure function; host only.
 *   partitionable  host [B] flags, or NULL = every block except the first of each stage
 *   sub_offsets    host [S+1] out: sub s owns sub_blocks[sub_offsets[s] .. sub_offsets[s+1])
 *   sub_blocks     host [cap] out: global block indices, ascending within a sub-ResNet
 *   owner_count    host [B] out: number of sub-ResNets holding each block (>= 1)
 * RESIST_EWORKSPACE if cap is too small (nothing is written past cap).
 */
int resist_partition(const resist_model_desc *desc, const uint8_t *partitionable, int32_t S,
                     int32_t min_depth, uint64_t seed, uint64_t round, int32_t *sub_offsets,
                     int32_t *sub_blocks, int32_t cap, int32_t *owner_count);

/* Size in floats of the parameter buffer of `block` (-1 stem, 0..B-1, B head): total, and the
 * trainable prefix that momentum / gradient buffers mirror.  host. */
int resist_block_param_count(const resist_model_desc *desc, int32_t block, int64_t *n_total,
                             int64_t *n_trainable);

/* Tensors inside the parameter buffer of `block`, in buffer order.  host.  Writes at most cap
 * entries and always the true number to *n_tensors. */
int resist_block_layout(const resist_model_desc *desc, int32_t block, resist_tensor_info *out,
                        int32_t cap, int32_t *n_tensors);

/* Bytes of device workspace resist_local_step needs for this sub-ResNet and batch size.  host. */
int resist_workspace_bytes(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks,
                           int32_t batch, int64_t *bytes);

/*
 * One local SGD iteration of one sub-ResNet on one batch (Algorithm 1, inner loop): forward,
 * backward (data and weight gradients), and the update  g += wd*w; v = mu*v + g; w -= lr*v  of
 * every trainable parameter the sub-ResNet holds.  Blocks not in `blocks` are not computed: the
 * residual stream passes through (Appendix B, mask = 0).  BN uses batch statistics (biased
 * variance) and updates the running statistics (unbiased variance, bn_momentum).
 *   blocks          host [nblocks] ascending global block indices; must contain the first block
 *                   of every stage
 *   block_params    host array [nblocks+2] of device fp32 buffers: stem, blocks..., head; updated
 *                   in place
 *   block_momentum  host array [nblocks+2] of device fp32 buffers (n_trainable floats each);
 *                   updated in place
 *   block_grads     NULL, or host array [nblocks+2] of device fp32 buffers (n_trainable floats
 *                   each) that receive dL/dW (before weight decay)
 *   x               device [batch,in_c,in_h,in_w] fp32;  labels: device [batch] int32 in
 *                   [0,num_classes)
 *   workspace       device, at least resist_workspace_bytes(); contents undefined afterwards
 *   loss_out        device, 1 float: mean cross-entropy of the batch (before the update)
 *   hip_stream      hipStream_t (NULL = default stream)
 */
int resist_local_step(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks,
                      void *const *block_params, void *const *block_momentum,
                      void *const *block_grads, const float *x, const int32_t *labels,
                      int32_t batch, float lr, float momentum, float weight_decay, void *workspace,
                      int64_t workspace_bytes, float *loss_out, void *hip_stream);

/*
 * Stream use of resist_local_step (not a step of the paper's method).  The weight-gradient kernels of
 * the backward pass, which only the parameter update at the end of the step needs (and likewise the
 * head's parameter gradients, the mean loss, and in the forward pass a block's shortcut convolution,
 * which the chain needs only at the block's end), can be enqueued
 * on a second stream the library creates per device (default priority, non-blocking), ordered
 * against hip_stream with events: started when their input is complete, joined before the update.
 * Seen from the caller everything is still ordered on hip_stream, and results are bit for bit the
 * same either way.
 *   mode 1 (default)  second stream for steps with at least ~20 GFLOP of convolution work (smaller
 *                     steps are bound by launch latency and the event calls would cost more)
 *   mode 2            second stream always
 *   mode 0            every kernel on hip_stream, one at a time (per-kernel timings are then those
 *                     of a kernel that has the GPU to itself)
 * Process-wide; takes effect at the next call.  host.
 */
int resist_set_overlap(int32_t mode);

/*
 * Where a step takes the first pass of a BN's backward (the per-channel sums of the output gradient
 * and of its product with the normalised input, Algorithm 1's dL/dW_s through every BN of a block).
 * A stride-1 data gradient can leave these sums per row tile from its epilogue while it stores the
 * gradient, instead of a separate pass that reads the gradient again.  Results agree with the
 * separate pass to fp32 rounding of the per-tile sums (the totals are added in float64 either way).
 *   mode 1 (default)  in bf16 steps (their backward chain, not the matrix cores, sets the step time)
 *   mode 2            in every step
 *   mode 0            never
 * Process-wide; takes effect at the next call.  host.
 */
int resist_set_bn_fusion(int32_t mode);

/*
 * Test-time forward pass (Sec. 2.6, "Scaling Activations"): logits of a batch through the stem, the
 * listed blocks and the head, with BN normalising by the running statistics stored in the block
 * buffers and the residual branch of blocks[i] multiplied by branch_scale[i] before the shortcut is
 * added:  out = ReLU(shortcut + branch_scale[i] * BN(last convolution of the branch)); for the
 * pre-activation kinds  out = shortcut + branch_scale[i] * (last convolution of the branch).  The paper
 * scales the partitioned blocks by 1/S when the reassembled global model uses all of them at once;
 * blocks every sub-ResNet trained get 1.  Nothing is written to the parameter buffers.
 *   blocks         host [nblocks] ascending, must contain the first block of every stage
 *   block_params   host array [nblocks+2] of device fp32 buffers: stem, blocks..., head
 *   branch_scale   host [nblocks] floats, or NULL = all 1
 *   x              device [batch,in_c,in_h,in_w] fp32
 *   workspace      device, at least resist_forward_workspace_bytes()
 *   logits_out     device [batch][num_classes] fp32
 *   labels, loss_out  both NULL, or device [batch] int32 and device 1 float (mean cross-entropy)
 */
int resist_forward_workspace_bytes(const resist_model_desc *desc, const int32_t *blocks,
                                   int32_t nblocks, int32_t batch, int64_t *bytes);
int resist_forward(const resist_model_desc *desc, const int32_t *blocks, int32_t nblocks,
                   void *const *block_params, const float *branch_scale, const float *x,
                   int32_t batch, void *workspace, int64_t workspace_bytes, float *logits_out,
                   const int32_t *labels, float *loss_out, void *hip_stream);

/*
 * Reassembly (Sec. 2.3; Appendix B: W = sum_v W_v M_v / sum_v M_v, last layer a = sum_v a_v / S):
 * every float of every block buffer of the global model (running statistics included) becomes the
 * mean over the sub-ResNets that hold the block -- fp32 sum in ascending sub-ResNet order, then one
 * division; a block held by one sub-ResNet is copied bit for bit; a block held by none is left
 * untouched.  Stem and head are averaged over all S.
 *   sub_offsets, sub_blocks   host, as written by resist_partition
 *   sub_block_params          host [S] arrays; sub_block_params[s] is a host array
 *                             [n_s + 2] of device buffers: stem, the blocks of s in order, head
 *   global_block_params       host array [B+2] of device buffers: stem, blocks 0..B-1, head
 * At most 16 sub-ResNets (S <= 16, the paper uses 2 to 8): more is RESIST_EUNSUPPORTED.
 */
int resist_aggregate(const resist_model_desc *desc, int32_t S, const int32_t *sub_offsets,
                     const int32_t *sub_blocks, void *const *const *sub_block_params,
                     void *const *global_block_params, void *hip_stream);

/*
 * Compressed communication (appendix "ResIST and Quantization/Sparse Gradients", Table 9: all
 * communicated parameters compressed to b bits, b = 8 ... 4).  The paper names no quantiser; the
 * library uses the uniform min-max one on every tensor of a block buffer separately:
 *     lo = min w, hi = max w, delta = (hi - lo) / (2^b - 1),
 *     code = round-half-even((w - lo) / delta) in 0 .. 2^b - 1   (all zero when delta == 0),
 *     decoded value lo + code * delta                          (fp32 throughout).
 * A compressed block is (a) a header of one resist_qrange per tensor, in the order of
 * resist_block_layout(), begin/end in floats from the start of the block buffer (alignment padding
 * between tensors belongs to no record: its code is 0 and it decodes to 0), and (b) one code per
 * float of the buffer: a byte each for b = 5..8; for b = 2..4 two per byte, float 2j in the low
 * nibble of byte j.
 *
 * resist_compressed_block_size: bytes of the code array and number of header records of `block`
 *   (-1 stem, 0..B-1, B head).  host.
 * resist_compress_blocks: compresses nkeys block buffers in a few launches.
 *   keys    host [nkeys] block keys (-1 stem, 0..B-1, B head)
 *   params  host [nkeys] device fp32 block buffers (read)
 *   codes   host [nkeys] device code arrays (written), 4-byte aligned
 *   ranges  host [nkeys] device arrays of n_tensors resist_qrange (written), 16-byte aligned
 * resist_aggregate_compressed: resist_aggregate with every source a compressed block: each float of
 *   the global model becomes the fp32 sum, in ascending sub-ResNet order, of the decoded copies times
 *   1/count (a single holder: its decoded copy; no holder: untouched).  sub_codes[s] / sub_ranges[s] are host
 *   arrays [n_s + 2] of device pointers laid out like sub_block_params of resist_aggregate; every
 *   copy must have been written by resist_compress_blocks with the same desc and bits.
 * resist_decompress_blocks: the other direction (server to worker): decodes nkeys compressed blocks
 *   into fp32 block buffers (every float lo + code * delta in one fp32 fused multiply-add, padding
 *   zero); arguments as for resist_compress_blocks with params written and codes, ranges read.
 * All are asynchronous on hip_stream; bits outside 2..8 is RESIST_EINVAL.
 */
typedef struct {
  float lo, delta;
  int32_t begin, end;
} resist_qrange;
int resist_compressed_block_size(const resist_model_desc *desc, int32_t block, int32_t bits,
                                 int64_t *code_bytes, int32_t *n_tensors);
int resist_compress_blocks(const resist_model_desc *desc, int32_t nkeys, const int32_t *keys,
                           int32_t bits, void *const *params, void *const *codes,
                           void *const *ranges, void *hip_stream);
int resist_decompress_blocks(const resist_model_desc *desc, int32_t nkeys, const int32_t *keys,
                             int32_t bits, void *const *codes, void *const *ranges,
                             void *const *params, void *hip_stream);
int resist_aggregate_compressed(const resist_model_desc *desc, int32_t S, const int32_t *sub_offsets,
                                const int32_t *sub_blocks, int32_t bits,
                                void *const *const *sub_codes, void *const *const *sub_ranges,
                                void *const *global_block_params, void *hip_stream);

/*
 * Optional per-kernel timing, for benchmarks (not a step of the paper's method).  While enabled,
 * every kernel launch is bracketed by two HIP events on the stream it is launched on.
 * resist_profile_enable(on) clears the statistics and switches timing on or off (off by default);
 * resist_profile_read waits for the recorded events and returns, per kernel, the number of launches,
 * the summed duration, and the summed algorithmic FLOPs and bytes of those launches.  Writes at
 * most cap entries and always the true number to *n.  host; not thread-safe against running steps.
 */
typedef struct {
  char name[64];
  int64_t launches;
  double ms;      /* summed launch durations (event to event)  */
  double flops;   /* summed algorithmic floating-point operations (2 per multiply-add) */
  double bytes;   /* summed algorithmic bytes read + written   */
} resist_kernel_stat;
int resist_profile_enable(int on);
int resist_profile_read(resist_kernel_stat *out, int32_t cap, int32_t *n);

/* Message for the last non-zero status returned on this thread (static storage). */
const char *resist_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RESIST_H */
