/*
 * sp3d.h -- C ABI of the spatially partitioned 3x3x3 convolution library for MI355X (gfx950).
 *
 * The operations are the steps of the paper's method (arxiv 1909.03108, Sec. 2, third
 * paragraph, and Fig. 1): a volume is cut into non-overlapping patches ("tiles"); before every
 * convolution each tile receives the margins ("halo", half the kernel size wide) of its
 * neighbours and is padded with them; then each tile is convolved on its own.  Forward and
 * backward of the convolutions are both on the path (Sec. 3, "Computational efficiency").
 * Here all tiles of the grid live in one GPU's memory and the exchange is an index mapping.
 *
 * General rules for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, at least 16-byte aligned.
 *     The library allocates nothing, frees nothing and keeps no state between calls except
 *     the code of the last HIP error (and the contents of the built-in scratch buffer of
 *     conv3d_wgrad_static, which no call relies on).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call checks
 *     its arguments on the host, enqueues its kernels on `stream` and returns without
 *     synchronising.
 *   - Return value: SP_OK (0) or a negative error code; on error nothing has been enqueued.
 *   - Geometry: volume extents (n, d, h, w); tile grid (gd, gh, gw) over the D, H, W axes, which
 *     must divide d, h, w; margin width `halo` of the padded layout.  Tile extents
 *     td = d/gd, th = h/gh, tw = w/gw; padded tile extents pd = td + 2*halo, etc.
 *     halo = 1 = floor(3/2) is what one 3x3x3 convolution needs (Sec. 2).  A wider margin lets a
 *     block of k <= halo convolutions run after ONE exchange of `halo`-wide margins, the overlap
 *     idea of Sec. 1 applied to a few layers: layer i of the block (i = 1..k) is called with
 *     grow = k - i and also computes the `grow` voxels around the interior that its successors
 *     read, instead of receiving them (redundant arithmetic in exchange for fewer exchanges).
 *     The grown box stops at the volume border: what lies beyond is zero padding at every layer.
 *   - 2-D variant (the paper's 2-D U-Net on slabs, Sec. 3: the same architecture with 2-D convolutions
 *     and poolings): with `flat` = 1 in the geometry the D axis is a stack of independent slices.  The
 *     convolutions then have extent 1 along D (weights w[3][3][Cin][Cout], taps (kh, kw)), the pooling
 *     and transposed-convolution windows are 1 x 2 x 2 (u[2][2][Cin][Cout]; the coarse side has
 *     extents d, h/2, w/2), a grown box does not grow along D, and the halo operations move only the
 *     8 regions with dd = 0.  The layouts are unchanged: the D margins of P and the other 18 regions
 *     of M exist but are neither read nor written.  Everything stated below for "3x3x3" / "2x2x2"
 *     holds with the D extent of the kernel or window set to 1.
 *
 * Layouts (C = channels, fastest)
 *   volume        V[n][d][h][w][C]
 *   padded tiles  P[n][gd][gh][gw][pd][ph][pw][C]; a tile's own voxels sit at [halo, halo+t) on
 *                 each axis ("interior"), the rest is its margin
 *   messages      M[n][gd][gh][gw][R][C], R = pd*ph*pw - td*th*tw; the R voxels of a tile are its
 *                 26 regions in lexicographic order of the direction (dd,dh,dw) in {-1,0,1}^3
 *                 without (0,0,0), each region row-major over its own (d,h,w) extents.  Region
 *                 `dir` holds the tile's own voxels nearest to the neighbour in direction `dir`:
 *                 on an axis with dir = -1 the first `halo` planes, +1 the last `halo`, 0 all.
 *   weights       w[3][3][3][Cin][Cout] in the tensor dtype (flat: w[3][3][Cin][Cout]); weight gradient
 *                 same shape, float
 *   bias          float[Cout]; bias gradient float[Cout]
 */
#ifndef SP3D_H
#define SP3D_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sp_geom {
    int32_t n, d, h, w;   /* whole-volume extents in voxels                     */
    int32_t gd, gh, gw;   /* tile grid over D, H, W; must divide d, h, w        */
    int32_t halo;         /* margin width of the layout, 1..SP_MAX_HALO          */
    int32_t grow;         /* conv3d_fwd*, conv3d_dgrad*: 0 <= grow < halo, see below; ignored elsewhere */
    int32_t flat;         /* 0: 3-D operations; 1: the 2-D variant (D = stack of slices), see above       */
    int32_t opts;         /* SP_HALO_* flags, see below; 0 = none                                           */
} sp_geom_t;

enum { SP_MAX_HALO = 4 };

typedef enum sp_dtype { SP_F32 = 0, SP_BF16 = 1 } sp_dtype_t;

enum {
    SP_OK = 0,
    SP_EINVAL = -1,        /* null pointer, misaligned pointer, non-positive extent/channels */
    SP_EGEOM = -2,         /* grid does not divide the volume, or a tile is thinner than halo */
    SP_EUNSUPPORTED = -3,  /* halo > SP_MAX_HALO, unknown dtype, channel count with no kernel */
    SP_EWORKSPACE = -4,    /* workspace missing or smaller than sp_workspace_bytes says       */
    SP_ELAUNCH = -5        /* HIP reported an error; see sp_last_hip_error()                  */
};

enum { SP_FLAG_RELU = 1 };                                /* conv3d_fwd: y = max(z, 0) */
/* sp_geom_t.opts.  A tile at the border of the volume has no neighbour in some directions: nothing it packs
 * for them is ever delivered, and the margins lying there are zero padding, not received data.
 *   SP_HALO_SKIP_SEND  halo_pack does not write the message regions that have no receiver (they keep whatever
 *                      they held).
 *   SP_HALO_KEEP_ZERO  halo_unpack and sp_halo_exchange do not write the margin regions at the volume border:
 *                      the caller guarantees that they hold zeros already.  A padded array that was zeroed once
 *                      stays that way, since no entry point writes margins beyond the volume border (the
 *                      convolutions with `grow` stop there too).
 *   SP_HALO_GATHER     conv3d_fwd*, conv3d_dgrad*, conv3d_wgrad*: the exchange fused into the convolution (Fig. 1b
 *                      and Sec. 2 with all tiles in one memory): wherever the call would read a margin voxel of
 *                      its input tensor that has a neighbour tile, it reads the voxel that the exchange would have
 *                      copied there - the neighbour's own voxel - so the input needs no halo_pack / halo_unpack /
 *                      sp_halo_exchange at all, and its margins towards neighbours are neither read nor written.
 *                      Margins at the volume border are read from the tensor and must hold zeros (as after
 *                      SP_HALO_KEEP_ZERO).  Same bits as the exchange followed by the plain call.  bf16 with
 *                      channel counts in multiples of 32, halo = 1, grow = 0, 3-D; the weight gradient also needs
 *                      tile extents along H and W in multiples of 8 and 32.  SP_EUNSUPPORTED otherwise (exchange
 *                      and call without the flag instead). */
enum { SP_HALO_SKIP_SEND = 1, SP_HALO_KEEP_ZERO = 2, SP_HALO_GATHER = 4 };
enum {                                                    /* sp_workspace_bytes `op`   */
    SP_OP_FWD = 0, SP_OP_DGRAD = 1, SP_OP_WGRAD = 2,      /* the 3x3x3 convolution     */
    SP_OP_UPCONV_WGRAD = 3,                               /* sp_upconv2_wgrad          */
    SP_OP_POINTWISE_WGRAD = 4,                            /* sp_pointwise_wgrad        */
    SP_OP_LOSS = 5                                        /* sp_dice_ce_loss: cin = classes, cout = 1 */
};

/* ---- host-only helpers (no GPU needed) --------------------------------------------------- */

/* Number of elements of the padded-tile array P / of the message array M for C channels;
 * 0 if the geometry is invalid. */
size_t sp_padded_elems(const sp_geom_t *g, int c);
size_t sp_msg_elems(const sp_geom_t *g, int c);
/* Bytes of scratch the convolution `op` needs for these sizes (may be 0); (size_t)-1 if the
 * combination is invalid or unsupported.  The size depends on the whole geometry (`grow` and `flat`
 * included): ask with the geometry that the call will get.  What a call leaves in the workspace is
 * of no use to the caller. */
size_t sp_workspace_bytes(int op, const sp_geom_t *g, int cin, int cout, sp_dtype_t dt);
/* 1 if conv3d_fwd* (op = SP_OP_FWD), conv3d_dgrad* (SP_OP_DGRAD) or conv3d_wgrad* (SP_OP_WGRAD) accepts
 * SP_HALO_GATHER for these sizes (g->opts itself is not looked at), else 0. */
int sp_gather_supported(int op, const sp_geom_t *g, int cin, int cout, sp_dtype_t dt);
/* SP_OK or the error the geometry would raise. */
int sp_check_geom(const sp_geom_t *g);
const char *sp_strerror(int code);
/* hipError_t of the most recent failing HIP call made by this library (0 if none). */
int sp_last_hip_error(void);

/* ---- partitioning (Fig. 1a; the "partitioning, reshaping" operations of Sec. 3) ------------ */

/* Copy every tile of V into the interior of its slot of P.  Margins of P are not written.
 * V and P must not overlap.  Bit-exact copy. */
int sp_partition(const void *vol, void *P, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream);
/* Inverse: drop the margins of P and reassemble V.  Bit-exact copy. */
int sp_unpartition(const void *P, void *vol, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream);

/* ---- halo exchange (Fig. 1b; Sec. 2: "exchange margins ... pad the patches") ---------------- */

/* Sending side: copy the 26 boundary regions of every tile's interior into its message (with
 * SP_HALO_SKIP_SEND: those that have a receiving tile).  Reads P's interiors only.  Bit-exact. */
int halo_pack(const void *P, void *msg, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream);
/* Receiving side: for every tile and direction `dir`, fill the margin region lying in direction
 * `dir` from region -dir of the message of the neighbour tile at +dir; zero-fill it when that
 * neighbour is outside the grid (zero 'same' padding at the volume border; with SP_HALO_KEEP_ZERO
 * such a region is left as it is).  Writes margins only; interiors are untouched.  P is updated in
 * place.  Bit-exact. */
int halo_unpack(void *P, const void *msg, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream);
/* halo_pack + delivery + halo_unpack in one pass for the case that all tiles live in one memory
 * (Sec. 2, Fig. 1b with the sending and the receiving device being the same): every margin region
 * of P is filled from the interior of the neighbour tile (zeros at the volume border), with no
 * message buffer.  Leaves P exactly as halo_pack followed by halo_unpack would.  In place. */
int sp_halo_exchange(void *P, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream);

/* ---- convolution on padded tiles (Sec. 2: "finally apply convolution"; Sec. 3: fwd + bwd) --- */

/* Forward.  z[v,co] = bias[co] + sum_{kd,kh,kw,ci} Px[v + (kd,kh,kw)][ci] * w[kd][kh][kw][ci][co]
 * for every interior voxel v of every tile (v in padded coordinates minus halo, so tap (1,1,1)
 * is the voxel itself): the 'valid' cross-correlation of each padded tile, which equals the
 * zero-padded 'same' convolution of the whole volume once halo_unpack has run on Px.
 * Writes y = z (or max(z,0) with SP_FLAG_RELU; of a NaN sum the result is NaN or, if its sign bit is set,
 * possibly zero) into the interiors of Py; Py's margins are left as they are.  bias may be NULL.  Px [..][Cin], Py [..][Cout] must not overlap.
 * With g->grow = e > 0 the output box of a tile is its interior plus e voxels on every side on which
 * the tile has a neighbour in the grid (the voxels the next e layers of a block read, computed here
 * instead of exchanged); Px must be valid e + 1 voxels around the interior.  The rest of Py's
 * margins is still left as it is: keep it zero beyond the volume border (a zeroed buffer stays so).
 * bf16: products of bf16 values accumulated in fp32, result rounded to nearest-even bf16.
 * f32: fp32 throughout.
 * bf16 layers whose Cin is not a multiple of 32 (but Cout is; Cin = 1 aside, which has kernels of its
 * own) run on the matrix cores through copies of Px and w with the channel axis zero-padded to the next
 * multiple of 32, held in `ws`: sp_workspace_bytes then asks for about one padded tensor of that many
 * channels.  conv3d_wgrad does the same and drops the padding rows of dw. */
int conv3d_fwd(const void *Px, const void *w, const float *bias, void *Py, const sp_geom_t *g,
               int cin, int cout, sp_dtype_t dt, uint32_t flags, void *ws, size_t ws_bytes,
               void *stream);

/* Data gradient.  dx[v,ci] = sum_{kd,kh,kw,co} Pdz[v + (2-kd,2-kh,2-kw)][co] * w[kd][kh][kw][ci][co]
 * over interior voxels v, i.e. the same correlation with the taps mirrored and the channel roles
 * swapped, reading halo-exchanged dz (run halo_pack/halo_unpack on Pdz first).  Writes the
 * interiors of Pdx [..][Cin] (with g->grow the grown box, as conv3d_fwd).  Precision as conv3d_fwd. */
int conv3d_dgrad(const void *Pdz, const void *w, void *Pdx, const sp_geom_t *g, int cin, int cout,
                 sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream);
/* Data gradient followed by the backward of the ReLU that produced this layer's input (Sec. 3: the
 * backward pass of a conv + ReLU stack):  Pdx[v,ci] = dx[v,ci] if Px[v,ci] > 0 else 0, with dx as in
 * conv3d_dgrad and Px [..][Cin] the layer's forward input (the previous layer's ReLU output).  Same
 * bits as conv3d_dgrad followed by sp_relu_bwd(Pdx, Px, Pdx), in one pass over Pdx.  Px must not
 * overlap Pdx. */
int conv3d_dgrad_relu(const void *Pdz, const void *w, const void *Px, void *Pdx, const sp_geom_t *g,
                      int cin, int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream);

/* ---- the ReLU mask as one bit per value ---------------------------------------------------
 * The backward pass of a conv + ReLU stack (Sec. 3) needs of a layer's input only whether each value was
 * positive.  Read as a tensor that is a second full pass over the activation; as bits it is 1/16 of it.
 * Layout of `bits` for a padded-tile array of C channels (C a multiple of 32; bf16): per padded voxel p
 * (index as in P, channels dropped) and block b of 32 channels two uint16_t words, at word index
 * (p * C/32 + b) * 2 + hi; word `hi` holds channel 32 b + 8 q + 4 hi + i in bit 4 q + i (q, i = 0..3).
 * (The order in which the matrix cores hand results to lanes, so that neither side shuffles.)
 * A bit is 1 where the value is positive - not zero, not negative, not NaN (conv3d_fwd_bits: a NaN result,
 * which its ReLU keeps only with a clear sign bit, gets a 1).  Only the words of interior
 * voxels mean anything: conv3d_fwd_bits leaves the others unwritten and no call reads them. */

/* Bytes of the bit array for C channels; 0 if the geometry or C is invalid. */
size_t sp_relu_bits_bytes(const sp_geom_t *g, int c);
/* 1 if conv3d_fwd_bits (op = SP_OP_FWD) / conv3d_dgrad_bits (SP_OP_DGRAD) runs for these sizes, else 0.
 * They serve the 3-D bf16 layers with channel counts in multiples of 32, and (forward) the first layer with
 * its single input channel; use the tensor forms elsewhere. */
int sp_relu_bits_supported(int op, const sp_geom_t *g, int cin, int cout, sp_dtype_t dt);
/* bits <- (Py > 0) for every padded voxel (margins included: whatever they hold). */
int sp_relu_bits(const void *Py, void *bits, const sp_geom_t *g, int c, sp_dtype_t dt, void *stream);
/* conv3d_fwd with SP_FLAG_RELU (which `flags` must hold) that also writes the bits of its result Py:
 * Py as from conv3d_fwd, bits as from sp_relu_bits(Py) at the interior voxels.  SP_EUNSUPPORTED where
 * sp_relu_bits_supported says 0. */
int conv3d_fwd_bits(const void *Px, const void *w, const float *bias, void *Py, void *bits, const sp_geom_t *g,
                    int cin, int cout, sp_dtype_t dt, uint32_t flags, void *ws, size_t ws_bytes, void *stream);
/* The same for the two-tensor forward pass conv3d_fwd2 (declared below; Cin = ca + cb). */
int conv3d_fwd2_bits(const void *Pxa, int ca, const void *Pxb, int cb, const void *w, const float *bias,
                     void *Py, void *bits, const sp_geom_t *g, int cout, sp_dtype_t dt, uint32_t flags,
                     void *ws, size_t ws_bytes, void *stream);
/* conv3d_dgrad_relu with the mask given as bits (of the layer's forward input, Cin channels) instead of
 * the tensor Px: the same bits in Pdx as conv3d_dgrad_relu with the Px that the bits were taken from. */
int conv3d_dgrad_bits(const void *Pdz, const void *w, const void *bits, void *Pdx, const sp_geom_t *g,
                      int cin, int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream);

/* Weight gradient.  dw[kd][kh][kw][ci][co] = sum over tiles and interior voxels v of
 * Px[v + (kd,kh,kw)][ci] * Pdz[v + (1,1,1)][co];  db[co] = sum of Pdz interiors (db may be NULL).
 * Px must hold its halos (as left by the forward pass); only the interiors of Pdz are read.
 * Products accumulated in fp32; the sum over workgroups is taken in a fixed order, so results
 * are reproducible run to run.  dw, db are float and are overwritten (not accumulated). */
int conv3d_wgrad(const void *Px, const void *Pdz, float *dw, float *db, const sp_geom_t *g,
                 int cin, int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream);

/* conv3d_wgrad for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the partial sums go to a buffer of
 * SP_STATIC_SCRATCH_BYTES that lives inside the library, one copy per GPU, held until the process ends.
 * Same arguments, same kernels and the same bits in dw / db as conv3d_wgrad.  The call allocates and frees
 * nothing; its first call on a device looks up that device's copy of the buffer (make that call outside a
 * graph capture).  SP_EWORKSPACE, with nothing enqueued, if sp_workspace_bytes(SP_OP_WGRAD, ...) for these
 * sizes exceeds SP_STATIC_SCRATCH_BYTES (32 MiB: enough for every layer with up to 512 x 512 channels).
 * Nothing in the buffer has to start at zero: every partial sum that the reduction reads is written by the
 * same call.  All calls on one GPU share the buffer: calls that overlap in time on one GPU (two streams, two
 * host threads) race; calls on one stream, one after the other, are safe. */
enum { SP_STATIC_SCRATCH_BYTES = 32 << 20 };
int conv3d_wgrad_static(const void *Px, const void *Pdz, float *dw, float *db, const sp_geom_t *g,
                        int cin, int cout, sp_dtype_t dt, void *stream);

/* The three passes on a channel-wise concatenation that is never materialised (the decoder of the
 * U-Net of Sec. 3 convolves concat(skip, up)): the layer's input channels [0, ca) live in tensor a
 * [..][ca] and [ca, ca + cb) in tensor b [..][cb]; w, dw are [3][3][3][ca + cb][Cout].  Results are
 * bit-identical to concatenating first and calling conv3d_fwd / conv3d_dgrad (+ split) / conv3d_wgrad.
 * bf16 with ca, cb, Cout multiples of 32 only (SP_EUNSUPPORTED otherwise: concatenate instead).
 * Workspace as for the single-tensor call with Cin = ca + cb.  Both inputs must hold their halos
 * (forward, weight gradient); conv3d_dgrad2 writes the interiors of both gradient tensors. */
int conv3d_fwd2(const void *Pxa, int ca, const void *Pxb, int cb, const void *w, const float *bias,
                void *Py, const sp_geom_t *g, int cout, sp_dtype_t dt, uint32_t flags, void *ws,
                size_t ws_bytes, void *stream);
int conv3d_dgrad2(const void *Pdz, const void *w, void *Pdxa, int ca, void *Pdxb, int cb,
                  const sp_geom_t *g, int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream);
int conv3d_wgrad2(const void *Pxa, int ca, const void *Pxb, int cb, const void *Pdz, float *dw,
                  float *db, const sp_geom_t *g, int cout, sp_dtype_t dt, void *ws, size_t ws_bytes,
                  void *stream);

/* Element-wise ReLU backward on padded tiles: Pdz = Pdy where Py > 0, else 0 (all elements,
 * margins included; the derivative at 0 is taken as 0).  Pdz may alias Pdy. */
int sp_relu_bwd(const void *Pdy, const void *Py, void *Pdz, const sp_geom_t *g, int c,
                sp_dtype_t dt, void *stream);

/* ---- U-Net glue around the convolutions (Sec. 3, first paragraph: blocks of convolutions with
 * max-pooling on the way down and a symmetric up-sampling path).  The paper names neither the
 * up-sampling operator nor the classifier; these are a 2x2x2 stride-2 transposed convolution, a
 * channel concatenation with the skip tensor and a 1x1x1 convolution.  Pooling / up-convolution
 * windows never straddle tiles, so none of these needs a halo; unless stated otherwise they read
 * and write tile interiors only and leave margins as they are.  "Fine" geometry `gf` = the
 * higher-resolution side (pool input, up-conv output); the coarse side has extents d/2, h/2, w/2 on
 * the same tile grid.  SP_EGEOM if a fine tile extent is odd. -------------------------------------- */

/* y[v,c] = max over the 2x2x2 window of Px starting at 2v.  Px fine [..][c], Py coarse [..][c]. */
int sp_maxpool2_fwd(const void *Px, void *Py, const sp_geom_t *gf, int c, sp_dtype_t dt, void *stream);
/* Pdx (fine) = Pdy (coarse) routed to the FIRST maximum of each window in (d,h,w) scan order, zero
 * for the other seven voxels.  Px is the pooling input. */
int sp_maxpool2_bwd(const void *Px, const void *Pdy, void *Pdx, const sp_geom_t *gf, int c,
                    sp_dtype_t dt, void *stream);
/* The backward pass of an encoder level of the network of Sec. 3 in one sweep.  The level's last ReLU
 * output Px (fine) feeds both the pooling and, as the skip tensor, the decoder; the gradient that
 * reaches the level's last convolution is therefore
 *     Pdz = [Px > 0] * (maxpool_bwd(Px, Pdy) + Pskip)
 * with Pdy (coarse) the gradient of the pooled tensor and Pskip (fine) the gradient that arrived through
 * the skip connection.  Same bits as sp_maxpool2_bwd, sp_add and sp_relu_bwd in that order (the sum in
 * fp32, rounded once).  Pskip may be the same tensor as Pdz; Px must not overlap Pdz. */
int sp_maxpool2_bwd_join(const void *Px, const void *Pdy, const void *Pskip, void *Pdz, const sp_geom_t *gf,
                         int c, sp_dtype_t dt, void *stream);

/* y[2v+(a,b,c), co] = bias[co] + sum_ci Px[v,ci] * u[a][b][c][ci][co];  u[2][2][2][Cin][Cout] in the
 * tensor dtype, bias float or NULL.  Px coarse [..][Cin], Py fine [..][Cout]. */
int sp_upconv2_fwd(const void *Px, const void *u, const float *bias, void *Py, const sp_geom_t *gf,
                   int cin, int cout, sp_dtype_t dt, void *stream);
/* dx[v,ci] = sum_{a,b,c,co} Pdy[2v+(a,b,c), co] * u[a][b][c][ci][co].  Pdy fine, Pdx coarse. */
int sp_upconv2_dgrad(const void *Pdy, const void *u, void *Pdx, const sp_geom_t *gf, int cin, int cout,
                     sp_dtype_t dt, void *stream);
/* du[a][b][c][ci][co] = sum_v Px[v,ci] * Pdy[2v+(a,b,c), co];  db[co] = sum Pdy (NULL to skip).
 * float outputs, overwritten; fixed-order reduction through `ws` (SP_OP_UPCONV_WGRAD). */
int sp_upconv2_wgrad(const void *Px, const void *Pdy, float *du, float *db, const sp_geom_t *gf,
                     int cin, int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream);

/* 1x1x1 convolution: y[v,co] = bias[co] + sum_ci Px[v,ci] * p[ci][co] (SP_FLAG_RELU allowed), its data
 * gradient dx[v,ci] = sum_co Pdy[v,co] * p[ci][co], and its weight / bias gradient (float, overwritten,
 * fixed-order reduction through `ws`, SP_OP_POINTWISE_WGRAD).  g is the geometry of both sides. */
int sp_pointwise_fwd(const void *Px, const void *p, const float *bias, void *Py, const sp_geom_t *g,
                     int cin, int cout, sp_dtype_t dt, uint32_t flags, void *stream);
int sp_pointwise_dgrad(const void *Pdy, const void *p, void *Pdx, const sp_geom_t *g, int cin, int cout,
                       sp_dtype_t dt, void *stream);
/* sp_pointwise_dgrad followed by the backward of the ReLU that produced the layer input Px [..][Cin]:
 * Pdx[v,ci] = dx[v,ci] if Px[v,ci] > 0 else 0, in one pass.  Px must not overlap Pdx. */
int sp_pointwise_dgrad_relu(const void *Pdy, const void *p, const void *Px, void *Pdx, const sp_geom_t *g,
                            int cin, int cout, sp_dtype_t dt, void *stream);
int sp_pointwise_wgrad(const void *Px, const void *Pdy, float *dp, float *db, const sp_geom_t *g,
                       int cin, int cout, sp_dtype_t dt, void *ws, size_t ws_bytes, void *stream);
/* The whole backward pass of a 1x1x1 layer whose input Px is a ReLU output, in one sweep over Px:
 * sp_pointwise_dgrad_relu (Pdx, same bits) and sp_pointwise_wgrad (dp, db - may be NULL -, same bits and
 * workspace, SP_OP_POINTWISE_WGRAD).  Px is read once instead of twice; shapes that the one-sweep kernel does
 * not serve (more than 4 output channels, Cin not a multiple of 8, fp32) run the two passes one after the
 * other.  Px must not overlap Pdx.  SP_EINVAL: p or Pdx NULL, overlap; SP_EWORKSPACE as sp_pointwise_wgrad. */
int sp_pointwise_bwd_relu(const void *Px, const void *Pdy, const void *p, void *Pdx, float *dp, float *db,
                          const sp_geom_t *g, int cin, int cout, sp_dtype_t dt, void *ws, size_t ws_bytes,
                          void *stream);

/* Channel concatenation Pout[..][ca+cb] = Pa[..][ca] ++ Pb[..][cb] and its inverse, over ALL voxels of
 * the padded arrays (margins included).  Bit-exact copies. */
int sp_concat(const void *Pa, int ca, const void *Pb, int cb, void *Pout, const sp_geom_t *g,
              sp_dtype_t dt, void *stream);
int sp_split(const void *Pin, void *Pa, int ca, void *Pb, int cb, const sp_geom_t *g, sp_dtype_t dt,
             void *stream);
/* Pout = Pa + Pb element-wise over all voxels of the padded arrays (the two gradient paths that meet
 * at a skip connection); fp32 addition, one rounding to the tensor dtype.  Pout may alias Pa or Pb. */
int sp_add(const void *Pa, const void *Pb, void *Pout, const sp_geom_t *g, int c, sp_dtype_t dt,
           void *stream);

/* ---- loss (Sec. 3, training set-up: 0.9 x Dice + 0.1 x cross-entropy; the paper gives no formula,
 *      the soft form of both terms is used) --------------------------------------------------------
 * p[v,:] = softmax of the logits of voxel v;  y = one-hot label;  V = all interior voxels of all tiles.
 *   Dice_c = (2 sum_v p[v,c] y[v,c] + eps) / (sum_v p[v,c] + sum_v y[v,c] + eps)
 *   loss   = w_dice (1 - mean_c Dice_c) - w_ce (1/V) sum_v log p[v, label v]
 * Plogits [..][classes] padded tiles; Plabels [..][1] padded tiles of the same dtype holding the class
 * index of every voxel (values outside [0, classes) are clamped); only interiors are read.
 * Outputs (each may be NULL, not all): Pdlogits [..][classes] = d loss / d logits, interiors written;
 * loss = 1 float; stats = 3*classes + 1 floats: sum p y, sum p, sum y per class, then -sum log p[label]
 * (the cross-tile sums; taken in a fixed order, so reproducible).  loss and stats are device pointers.
 * classes 2..4.  Workspace: sp_workspace_bytes(SP_OP_LOSS, g, classes, 1, dt). */
int sp_dice_ce_loss(const void *Plogits, const void *Plabels, void *Pdlogits, float *loss, float *stats,
                    const sp_geom_t *g, int classes, sp_dtype_t dt, float w_dice, float w_ce, float eps,
                    void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SP3D_H */
