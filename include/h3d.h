/*
 * h3d — per-GPU hot path of spatially-partitioned ("hybrid-parallel") 3-D CNN
 * training on AMD MI355X (gfx950): dense 3x3x3 convolution forward /
 * backward-data / backward-filter with fused bias and (leaky-)ReLU, 2x2x2
 * pooling, and halo pack/unpack, on one GPU's depth slab of an N,C,D,H,W
 * sample (paper Sec. II-B "spatial partitioning", Sec. III-A, Sec. III-C).
 *
 * Plain C ABI.  No C++ types, no exceptions, no torch types.
 *
 * POINTERS.  Every `data`, weight, bias, gradient, buffer and workspace pointer
 * is a DEVICE pointer owned by the caller (for instance a torch tensor's
 * data_ptr()).  Descriptor structs (`h3d_tensor`) and the handle are HOST memory.
 * The library never allocates or frees device memory; scratch space is passed
 * in as a workspace whose size is queried with h3d_*_workspace_bytes.
 *
 * ASYNCHRONY.  Every compute call only enqueues kernels on `stream`
 * (a hipStream_t passed as void*; NULL = the default stream) and returns.
 *
 * ERRORS.  Every call returns an h3d_status.  Argument violations are found on
 * the host BEFORE anything is launched; nothing aborts or throws.
 * h3d_last_error(handle) gives a human-readable reason for the last failure
 * on that handle.
 *
 * TENSORS.  N,C,D,H,W, fully packed, W fastest (paper Sec. III "Notation").
 * A slab stores halo_lo + d + halo_hi depth planes per (n,c).  Interior plane
 * p in [0,d) is global plane d_offset + p of a sample whose unsharded depth is
 * d_global; halo plane p in [-halo_lo,0) or [d,d+halo_hi) holds the
 * neighbouring shard's boundary data (Sec. II-B: halo exchange).  Everything
 * outside the global volume [0,d_global) x [0,h) x [0,w) is zero ("same"
 * padding, Table I caption) and is never read, whatever the halo planes there
 * contain.  An unsharded tensor is the case halo 0, d_offset 0, d_global = d.
 * H and W are not partitioned (the paper evaluates depth partitioning, Sec. V).
 */
#ifndef H3D_H
#define H3D_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { H3D_F32 = 0, H3D_BF16 = 1 } h3d_dtype;

typedef enum {
  H3D_OK = 0,
  H3D_EINVAL = -1,       /* NULL pointer, shape/dtype mismatch, bad enum            */
  H3D_EUNSUPPORTED = -2, /* valid request this build has no kernel for              */
  H3D_EWORKSPACE = -3,   /* workspace NULL or smaller than h3d_*_workspace_bytes    */
  H3D_EHALO = -4,        /* a needed plane inside the global volume is not stored   */
  H3D_EHIP = -5          /* HIP runtime error on launch                             */
} h3d_status;

typedef enum { H3D_ACT_NONE = 0, H3D_ACT_RELU = 1, H3D_ACT_LEAKY = 2 } h3d_act;
typedef enum { H3D_POOL_AVG = 0, H3D_POOL_MAX = 1 } h3d_pool;
/* D_BOTH: the two depth faces in one call (one launch instead of two: the faces of a shard are small, and a call costs a
 * kernel launch whatever its size); the buffer then holds the LO face followed by the HI face, h3d_halo_bytes each. */
typedef enum { H3D_FACE_D_LO = 0, H3D_FACE_D_HI = 1, H3D_FACE_D_BOTH = 2 } h3d_face;
typedef enum { H3D_OP_FWD = 0, H3D_OP_BWD_DATA = 1, H3D_OP_BWD_FILTER = 2 } h3d_conv_op;

typedef struct {
  void* data;               /* DEVICE pointer to [n][c][halo_lo+d+halo_hi][h][w]          */
  int32_t dtype;            /* h3d_dtype                                                   */
  int32_t n, c;             /* samples, channels                                           */
  int32_t d, h, w;          /* INTERIOR extents of this shard                              */
  int32_t halo_lo, halo_hi; /* stored halo planes below / above the interior              */
  int64_t d_offset;         /* global depth index of interior plane 0                      */
  int64_t d_global;         /* depth of the unsharded sample                               */
  /* Elements between consecutive channels / samples.  0 = packed: (halo_lo+d+halo_hi)*h*w and c times that.
   * Non-zero strides describe a VIEW of a larger stored tensor: a RUN OF PLANES inside a taller slab, i.e. the main /
   * halo sub-domains of Sec. III-C (D_main = planes that need no halo, D_halo = the strips that do), and / or a RANGE
   * OF CHANNELS of a tensor with more channels (the two halves of a U-Net concatenation, Sec. III-A: a layer then
   * writes its output straight into its half and no copy is made).  `data` points at the view's first stored plane
   * of its first channel, n / c / d / halo_* / d_offset describe the view, the strides are the parent's.  Views are
   * accepted by the three convolution passes, h3d_act_bwd, h3d_pool3d_fwd / _bwd / _bwd_act and the h3d_deconv2_*
   * calls; every other entry point returns H3D_EUNSUPPORTED.
   * Forward / backward-data on views that tile a slab give the whole-slab call's result bit for bit, except
   * where the whole-slab call is small enough to take the channel-split kernel (bf16, W <= 16, fewer than 64
   * workgroups): views are never split, so the fp32 summation order of the two differs there. */
  int64_t c_stride;
  int64_t n_stride;
} h3d_tensor;

/* Handle: host object caching device properties and the last error text.
 * Not thread-safe; use one per host thread.  Bound to the device current at creation. */
h3d_status h3d_create(void** handle);
h3d_status h3d_destroy(void* handle);
const char* h3d_last_error(void* handle); /* handle-owned string, valid until the next call */
/* For measurement tools: the name of the kernel that did the arithmetic of the last successful compute call on this
 * handle (a call may also launch small helper kernels: weight packing, the ordered second stage of a reduction), as a
 * profiler's kernel trace spells it, template arguments included where the library chooses among instances; "" before
 * the first call.  Handle-owned string, valid until the next call. */
const char* h3d_last_kernel(void* handle);

/* ---- 3x3x3 convolution, stride 1, zero padding 1 (Table I caption; FP/BD/BF of Sec. III-C) ----
 *
 * Weights w: [cout][cin][3][3][3] packed, same dtype as the activations.
 * bias: fp32 [cout] or NULL (the paper's CosmoFlow variant drops conv biases, Sec. IV).
 * act/alpha: z = y > 0 ? y : slope*y with slope = alpha (LEAKY), 0 (RELU), 1 (NONE).
 *
 * Workspace bytes needed by `op` for these shapes (0 is possible).  Returns 0 on bad arguments. */
size_t h3d_conv3d_workspace_bytes(void* handle, int op, const h3d_tensor* x, const h3d_tensor* z);

/* Forward: z[n,co,p] = act(bias[co] + sum_{ci,kd,kh,kw} w[co,ci,kd,kh,kw] * x~[n,ci,p+k-1])
 * (cross-correlation) for every stored plane p of z, i.e. p in [-z.halo_lo, d+z.halo_hi):
 * a z with halos asks for "halo recompute" and needs x to store one plane more on that side.
 * Planes of z outside the global volume are written as ZERO (they are the next layer's padding).
 * x and z must agree in n,d,h,w,d_offset,d_global,dtype.  H3D_EHALO if x lacks a needed plane. */
h3d_status h3d_conv3d_fwd(void* handle, const h3d_tensor* x, const void* w, const float* bias,
                          h3d_tensor* z, int act, float alpha, void* ws, size_t ws_bytes, void* stream);

/* Backward-data: g = dz * (z > 0 ? 1 : slope) with z the saved forward OUTPUT
 * (z == NULL or act NONE: g = dz);  dx[n,ci,q] = sum_{co,k} w[co,ci,k] * g~[n,co,q-k+1]
 * for every stored plane q of dx.  dz (and z) must store the planes q-1..q+1 that lie inside
 * the volume (their halos come from the neighbours by halo exchange), else H3D_EHALO. */
h3d_status h3d_conv3d_bwd_data(void* handle, const h3d_tensor* dz, const h3d_tensor* z, const void* w,
                               h3d_tensor* dx, int act, float alpha, void* ws, size_t ws_bytes, void* stream);

/* Backward-filter: dw[co,ci,k] = sum_n sum_{p in interior} g[n,co,p] * x~[n,ci,p+k-1], db[co] = sum g.
 * dw fp32 [cout][cin][3][3][3] and db fp32 [cout] (or NULL) are OVERWRITTEN with this shard's
 * partial gradient (the sum over shards and data-parallel replicas is the allreduce of Sec. III-A,
 * outside this library).  Deterministic: a fixed split of the voxel range and a fixed-order second
 * stage, so two calls with the same inputs return identical bits. */
h3d_status h3d_conv3d_bwd_filter(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z,
                                 float* dw, float* db, int act, float alpha, void* ws, size_t ws_bytes,
                                 void* stream);

/* ---- backward-filter without a workspace argument and without any allocation ----
 * For callers that cannot allocate device memory or size a workspace: code under HIP graph capture, tight serving /
 * training loops, harnesses that forbid hipMalloc.  Same arguments, kernels, results (bit for bit) and errors as
 * h3d_conv3d_bwd_filter; the per-chunk partial sums of the split-spatial reduction go to a device array of
 * h3d_static_scratch_bytes() bytes (96 MiB) that the library owns: one copy per GPU it runs on, held until the process
 * ends, its address looked up once per device by h3d_create.  Shapes whose h3d_conv3d_workspace_bytes(BWD_FILTER)
 * exceeds that size are rejected with H3D_EWORKSPACE before anything is launched (then use the call above).  The call
 * allocates and frees nothing, on the host or the device, and does not synchronise.  Every call on a GPU shares that
 * GPU's array: calls that overlap in time on one GPU (two streams, two threads) race and must be serialised by the
 * caller; nothing needs to be cleared between calls (the second stage reads only what the first stage of the same call
 * wrote).  The handle must belong to the current device (H3D_EINVAL otherwise). */
size_t h3d_static_scratch_bytes(void);
h3d_status h3d_conv3d_bwd_filter_static(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z,
                                        float* dw, float* db, int act, float alpha, void* stream);

/* ---- 3x3x3 convolution with a stride of 2 (Table I: the fourth convolution of the CosmoFlow network) ----
 * "Same" padding is read as one zero voxel on every side, as for the stride-1 layers, so an even extent is halved
 * (an odd h or w is rounded up):  y[n,co,p] = act(bias[co] + sum_{ci,k} w[co,ci,k] * x~[n,ci,2p+k-1]).
 * x: the input shard, d, d_offset and d_global even (else H3D_EUNSUPPORTED: an output voxel would belong to two
 * shards); y: the output shard, n equal, d/2, ceil(h/2), ceil(w/2), d_offset/2, d_global/2.  Packed tensors only;
 * weights, bias, dw, db, act as for the stride-1 calls.  Interiors are written; halo planes of the OUTPUT argument
 * of each call are neither read nor written.  Which halo planes are READ differs by direction:
 *   forward, backward-filter: output plane p reads input planes 2p-1 .. 2p+1, so x needs its LOWER halo plane
 *     (when inside the volume), never the upper one;
 *   backward-data: input plane d-1 receives a term from output plane d/2, so dy (and y, when act is not NONE)
 *     need their UPPER halo plane, never the lower one.                                  H3D_EHALO otherwise.
 * Workspace: h3d_conv3d_s2_workspace_bytes(handle, op, x, y) with x / y the input-side / output-side descriptors
 * for every op; 256-byte aligned.  The call rewrites the problem as a stride-1 convolution over the eight parity
 * sub-lattices of x and runs the stride-1 kernels; the workspace holds the rearranged tensors. */
size_t h3d_conv3d_s2_workspace_bytes(void* handle, int op, const h3d_tensor* x, const h3d_tensor* y);
h3d_status h3d_conv3d_s2_fwd(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* y,
                             int act, float alpha, void* ws, size_t ws_bytes, void* stream);
/* g = dy * (y > 0 ? 1 : slope);  dx[n,ci,q] = sum over (co,k,p) with 2p+k-1 = q of w[co,ci,k] * g[n,co,p]. */
h3d_status h3d_conv3d_s2_bwd_data(void* handle, const h3d_tensor* dy, const h3d_tensor* y, const void* w,
                                  h3d_tensor* dx, int act, float alpha, void* ws, size_t ws_bytes, void* stream);
/* dw[co,ci,k] = sum_n sum_{p in the output shard} g[n,co,p] * x~[n,ci,2p+k-1], db[co] = sum g; overwritten;
 * deterministic like h3d_conv3d_bwd_filter. */
h3d_status h3d_conv3d_s2_bwd_filter(void* handle, const h3d_tensor* x, const h3d_tensor* dy, const h3d_tensor* y,
                                    float* dw, float* db, int act, float alpha, void* ws, size_t ws_bytes,
                                    void* stream);

/* ---- 5x5x5 convolution, stride 1, zero padding 2 (Sec. III-A: 3^3 and 5^3 are the filter sizes the halo packing
 * kernels are specialised for; with 5^3 the halo is two planes wide) ----
 * Weights w: [cout][cin][5][5][5] packed, same dtype as the activations; bias, dw ([cout][cin][5][5][5] fp32), db,
 * act / alpha as for the 3x3x3 calls.  Packed tensors only; both descriptors of a call are the same shard (n, d, h, w,
 * d_offset, d_global, dtype) with at least one channel each.  The shard INTERIOR of the output argument is written;
 * its halo planes are neither read nor written.  The tensor a call reads through the window (x in forward and
 * backward-filter; dz, and z when act is not NONE, in backward-data) must store min(2, planes of the volume on that
 * side) halo planes below and above, else H3D_EHALO; planes outside the global volume count as zero.
 *   forward:          z[n,co,p]  = act(bias[co] + sum_{ci,k} w[co,ci,k] * x~[n,ci,p+k-2])
 *   backward-data:    dx[n,ci,q] = sum_{co,k} w[co,ci,k] * g~[n,co,q-k+2],  g = dz * (z > 0 ? 1 : slope)
 *   backward-filter:  dw[co,ci,k] = sum_n sum_{p in the interior} g[n,co,p] * x~[n,ci,p+k-2],  db[co] = sum g
 *                     (overwritten; the shard's partial gradient; deterministic: fixed chunks of tiles, added in order)
 * Workspace: h3d_conv3d_k5_workspace_bytes(handle, op, x, z) with x / z the input-side / output-side descriptors for
 * every op (packed copy of the filter, or the per-chunk partial sums; for bf16 backward passes also g = dz * act'(z),
 * the size of dz); 256-byte aligned; H3D_EWORKSPACE if too small.
 * More than 65535 interior planes or n * ceil(channels/16) > 65535: H3D_EUNSUPPORTED.  fp32 accumulation; bf16
 * tensors run on the matrix cores (backward-data and backward-filter then round g to bf16 once, as the 3x3x3 calls
 * do; backward-filter needs w a multiple of 8 and 16-byte aligned data for that form), fp32 tensors and the
 * remaining bf16 cases on the vector ALU. */
size_t h3d_conv3d_k5_workspace_bytes(void* handle, int op, const h3d_tensor* x, const h3d_tensor* z);
h3d_status h3d_conv3d_k5_fwd(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* z,
                             int act, float alpha, void* ws, size_t ws_bytes, void* stream);
h3d_status h3d_conv3d_k5_bwd_data(void* handle, const h3d_tensor* dz, const h3d_tensor* z, const void* w,
                                  h3d_tensor* dx, int act, float alpha, void* ws, size_t ws_bytes, void* stream);
h3d_status h3d_conv3d_k5_bwd_filter(void* handle, const h3d_tensor* x, const h3d_tensor* dz, const h3d_tensor* z,
                                    float* dw, float* db, int act, float alpha, void* ws, size_t ws_bytes,
                                    void* stream);

/* ---- activation backward as a separate pass (Sec. IV: leaky-ReLU after every conv; U-Net: ReLU) ----
 * g = (dz + dz2) * (z > 0 ? 1 : slope) on the shard INTERIOR; dz2 may be NULL (it merges the two
 * gradient branches of a skip connection).  z is the saved forward output.  Halo planes of g are
 * not written: they are filled by the backward halo exchange, after which the backward
 * convolutions are called with act NONE.  All tensors agree in n,c,d,h,w,offsets,dtype; halos may differ. */
h3d_status h3d_act_bwd(void* handle, const h3d_tensor* dz, const h3d_tensor* dz2, const h3d_tensor* z,
                       h3d_tensor* g, int act, float alpha, void* stream);

/* ---- 2x2x2 stride-2 pooling of the shard interior (Table I: stride-2 pooling; Sec. III-A) ----
 * y interior extents are x's halved; d, h, w and d_offset of x must be even so that no window
 * straddles a shard face (else H3D_EUNSUPPORTED).  Halo planes of x and y are neither read nor
 * written.  AVG: mean of 8.  MAX: maximum of 8. */
h3d_status h3d_pool3d_fwd(void* handle, const h3d_tensor* x, h3d_tensor* y, int mode, void* stream);
/* AVG: dx[2q+k] = dy[q]/8.  MAX: dy[q] goes to the FIRST maximal element of the window of x (the
 * forward input, required) in (kd,kh,kw) row-major order, zero to the other seven. */
h3d_status h3d_pool3d_bwd(void* handle, const h3d_tensor* dy, const h3d_tensor* x, h3d_tensor* dx, int mode,
                          void* stream);

/* Pooling backward fused with the activation backward of the layer below it:
 * g = (pool3d_bwd(dy) + dz2) * (z > 0 ? 1 : slope), z the saved output of the conv+activation that fed the
 * pooling (same shape as g; its halos may differ); dz2 (same shape as g, or NULL) is a second gradient arriving at
 * that output - the skip branch of a U-Net level (Sec. III-A), which leaves the encoder beside the pooling.  One
 * streaming pass instead of pooling backward, add and activation backward; the backward convolutions are then called
 * on g with act NONE.  The un-pooled gradient is rounded to the storage type as h3d_pool3d_bwd stores it, then the
 * sum is masked and rounded once: the bits of the separate calls. */
h3d_status h3d_pool3d_bwd_act(void* handle, const h3d_tensor* dy, const h3d_tensor* x, const h3d_tensor* z,
                              const h3d_tensor* dz2, h3d_tensor* g, int mode, int act, float alpha, void* stream);

/* ---- convolution forward fused with the 2x2x2 average pooling that follows it, and the matching backward step ----
 * (Sec. III-A: operations that are "normally considered cheap" - pooling, activations - dominate once the tensors
 * are large; here the unpooled activation never has to travel to memory and back.)
 * AVERAGE pooling only (the CosmoFlow shapes; a max-pooled layer uses the separate calls).
 * y = avgpool(act(b + W * x)): the pooled tensor of the same shard (extents and offsets half of z's, halos allowed,
 * interior written).  z describes the unpooled output; z->data == NULL means it is not stored (only where a fused
 * kernel exists: bf16, Cin <= 4, Cout <= 32, z without halos, even d and h, w a multiple of 8; otherwise
 * H3D_EUNSUPPORTED) - with z->data set the call works for every shape h3d_conv3d_fwd and h3d_pool3d_fwd accept.
 * mask (DEVICE, h3d_act_mask_bytes(z) bytes, or NULL): one bit per unpooled voxel, set where the stored output is
 * > 0; bit k of byte j of a row is voxel 8 j + k, rows packed [n][c][interior plane][h][w/8].  It replaces z in
 * the backward pass (1/16 of its bytes).  A mask with w not a multiple of 8 is H3D_EUNSUPPORTED, found before any launch. */
size_t h3d_act_mask_bytes(const h3d_tensor* z);                       /* 0 if w is not a multiple of 8 */
h3d_status h3d_conv3d_fwd_pool(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* z,
                               h3d_tensor* y, void* mask, int act, float alpha,
                               void* ws, size_t ws_bytes, void* stream);
/* mask of a stored output z (what the fused call writes by itself). */
h3d_status h3d_act_mask(void* handle, const h3d_tensor* z, void* mask, void* stream);
/* y = avgpool(x) and, in the same pass, the mask of x (what h3d_pool3d_fwd and h3d_act_mask write one after the other):
 * for the layers whose activation IS stored, so that their backward pass need not read it again.  bf16, w a multiple
 * of 16, 32-byte-aligned x; otherwise H3D_EUNSUPPORTED. */
h3d_status h3d_pool3d_fwd_mask(void* handle, const h3d_tensor* x, h3d_tensor* y, void* mask, void* stream);
/* g = avgpool_bwd(dy) * (bit ? 1 : slope): h3d_pool3d_bwd_act with the mask in place of z; same bits in g.
 * bf16, w a multiple of 16, act RELU or LEAKY. */
h3d_status h3d_pool3d_bwd_mask(void* handle, const h3d_tensor* dy, const void* mask, h3d_tensor* g, int act, float alpha,
                               void* stream);

/* ---- halo pack / unpack of the depth faces (Sec. III-A: packing/unpacking kernels for the
 *      neighbour communication of boundary regions) ---- bit-exact copies.
 * Face buffer layout: [n][c][width][h][w] packed, same dtype as t. */
size_t h3d_halo_bytes(const h3d_tensor* t, int width);
/* pack: copy the `width` outermost INTERIOR planes at `face` into buf (what the neighbour needs).
 * face D_BOTH: buf = [LO face][HI face], 2 * h3d_halo_bytes(t, width) bytes. */
h3d_status h3d_halo_pack(void* handle, const h3d_tensor* t, int face, int width, void* buf, void* stream);
/* unpack: write buf into the `width` HALO planes adjacent to the interior at `face`
 * (width <= that halo); buf == NULL zero-fills them (global boundary).
 * face D_BOTH: buf = [planes for the LO halo][planes for the HI halo] (width <= both halos); NULL zero-fills both. */
h3d_status h3d_halo_unpack(void* handle, const void* buf, h3d_tensor* t, int face, int width, void* stream);

/* ---- general faces (Sec. II-B: the spatial domain may be partitioned in any of its three dimensions;
 *      Sec. III-A: packing / unpacking kernels of the boundary exchange for 3^3 and 5^3 filters, i.e. faces
 *      one or two voxels wide) ---- bit-exact copies.
 * t: DEVICE pointer to a packed tensor [n][c][D][H][W] of `dtype`; D, H, W are its STORED extents (the
 * caller decides which planes, rows and columns of it are halo).  box: origin (d0,h0,w0) and extents
 * (bd,bh,bw) of the face inside every (n,c) volume; buf: DEVICE pointer to [n][c][bd][bh][bw] packed.
 * Nothing is allocated or owned; a box that does not lie inside the tensor is H3D_EINVAL before any launch;
 * an empty box is a no-op. */
typedef struct {
  int32_t d0, h0, w0;   /* origin of the box */
  int32_t bd, bh, bw;   /* extents of the box */
} h3d_box;
size_t h3d_box_bytes(int dtype, int n, int c, const h3d_box* box);
/* pack: buf <- box of t. */
h3d_status h3d_box_pack(void* handle, const void* t, int dtype, int n, int c, int D, int H, int W,
                        const h3d_box* box, void* buf, void* stream);
/* unpack: box of t <- buf; buf == NULL writes zeros (a face on the global boundary).  Elements of t
 * outside the box are not touched. */
h3d_status h3d_box_unpack(void* handle, const void* buf, void* t, int dtype, int n, int c, int D, int H, int W,
                          const h3d_box* box, void* stream);

/* ---- 2x2x2 stride-2 transposed convolution (U-Net up-sampling "deconvolution", Sec. III-A) ----
 * w: [cin][cout][2][2][2]; y[n,co,2q+k] = bias[co] + sum_ci w[ci,co,k] * x[n,ci,q].  Interiors only;
 * y interior extents are twice x's. */
size_t h3d_deconv2_workspace_bytes(void* handle, int op /* h3d_conv_op */, const h3d_tensor* x, const h3d_tensor* y);
h3d_status h3d_deconv2_fwd(void* handle, const h3d_tensor* x, const void* w, const float* bias, h3d_tensor* y,
                           void* ws, size_t ws_bytes, void* stream);
/* dx[n,ci,q] = sum_{co,k} w[ci,co,k] * dy[n,co,2q+k] */
h3d_status h3d_deconv2_bwd_data(void* handle, const h3d_tensor* dy, const void* w, h3d_tensor* dx, void* ws,
                                size_t ws_bytes, void* stream);
/* dw[ci,co,k] = sum_{n,q} x[n,ci,q] * dy[n,co,2q+k], db[co] = sum dy: dw fp32 [cin][cout][2][2][2] and
 * db fp32 [cout] (or NULL) are overwritten; deterministic (fixed split + fixed-order second stage). */
h3d_status h3d_deconv2_bwd_filter(void* handle, const h3d_tensor* x, const h3d_tensor* dy, float* dw, float* db,
                                  void* ws, size_t ws_bytes, void* stream);

/* ---- channel concat / split of interiors (U-Net skip connections, Sec. III-A) ---- bit-exact.
 * out channels [0,a.c) = a, [a.c, a.c+b.c) = b.  split is the inverse (the backward of concat). */
h3d_status h3d_concat_c(void* handle, const h3d_tensor* a, const h3d_tensor* b, h3d_tensor* out, void* stream);
h3d_status h3d_split_c(void* handle, const h3d_tensor* in, h3d_tensor* a, h3d_tensor* b, void* stream);

/* ---- fully-connected layers and the MSE loss that close the CosmoFlow stack (Table I, Sec. IV) ----
 * x [m][k], w [n][k] (dtype of x), bias fp32 [n] or NULL, y [m][n] (dtype of x): y = act(x w^T + bias).
 * m <= 8 rows per call (the per-GPU sample count after the spatial layers), else H3D_EUNSUPPORTED. */
h3d_status h3d_dense_fwd(void* handle, const void* x, const void* w, const float* bias, void* y, int dtype, int m,
                         int n, int k, int act, float alpha, void* stream);
/* dy [m][n], y saved output; dx [m][k] (dtype) or NULL, dw fp32 [n][k] or NULL, db fp32 [n] or NULL (NULL when dw
 * is NULL); overwritten.  The two halves are independent kernels: a caller may ask for dx alone and for dw / db
 * alone in two calls (on two streams). */
h3d_status h3d_dense_bwd(void* handle, const void* x, const void* w, const void* y, const void* dy, void* dx,
                         float* dw, float* db, int dtype, int m, int n, int k, int act, float alpha, void* stream);
/* loss[0] (fp32, device) = mean over all `count` entries of (pred-target)^2; dpred = 2 (pred-target)/count
 * (dtype of pred); target fp32.  count <= 65536. */
h3d_status h3d_mse_fwd_bwd(void* handle, const void* pred, const float* target, float* loss, void* dpred, int dtype,
                           int count, void* stream);

/* ---- batch normalisation, the parts local to a shard (Sec. II-B: partial statistics per partition are aggregated
 * with an allreduce; Sec. III-C: a batch-normalisation layer costs this computation plus the allreduce of the
 * per-channel sum and squared sum).  The allreduce itself is the caller's.  All per-channel arrays are fp32
 * device memory of x->c entries; sums run over the INTERIOR planes of the slab only, in a fixed order (the
 * same inputs give the same bits); halo planes are neither read nor written.  Packed tensors only.
 * Workspace: h3d_bn_workspace_bytes(x) bytes for every call below that takes one. */
size_t h3d_bn_workspace_bytes(void* handle, const h3d_tensor* x);
/* sum[c] = sum of x, sqsum[c] = sum of x^2 over n, d, h, w of this shard. */
h3d_status h3d_bn_stats(void* handle, const h3d_tensor* x, float* sum, float* sqsum, void* ws, size_t ws_bytes, void* stream);
/* mean = sum / count, invstd = 1 / sqrt(sqsum / count - mean^2 + eps) (biased variance, clamped at 0), from the
 * statistics summed over all shards; count = voxels per channel over all shards and samples. */
h3d_status h3d_bn_finalize(void* handle, const float* sum, const float* sqsum, int channels, int64_t count, float eps,
                           float* mean, float* invstd, void* stream);
/* y = gamma * (x - mean) * invstd + beta on the interior (gamma / beta NULL = 1 / 0); y: same shard as x. */
h3d_status h3d_bn_fwd(void* handle, const h3d_tensor* x, const float* mean, const float* invstd, const float* gamma,
                      const float* beta, h3d_tensor* y, void* ws, size_t ws_bytes, void* stream);
/* sum_dy[c] = sum of dy (the shard's part of dbeta), sum_dy_xhat[c] = sum of dy * (x - mean) * invstd (of dgamma). */
h3d_status h3d_bn_bwd_stats(void* handle, const h3d_tensor* dy, const h3d_tensor* x, const float* mean, const float* invstd,
                            float* sum_dy, float* sum_dy_xhat, void* ws, size_t ws_bytes, void* stream);
/* dx = gamma * invstd * (dy - sum_dy / count - xhat * sum_dy_xhat / count), with the two sums taken over all shards. */
h3d_status h3d_bn_bwd(void* handle, const h3d_tensor* dy, const h3d_tensor* x, const float* mean, const float* invstd,
                      const float* gamma, const float* sum_dy, const float* sum_dy_xhat, int64_t count, h3d_tensor* dx,
                      void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* H3D_H */
