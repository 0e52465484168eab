"""Forward + backward of the 3D U-Net convolution stack on a tile grid, as a sequence of C-ABI calls.

Plumbing only: this module allocates device buffers (torch) and orders the library calls; every
operation -- partition, halo exchange, the convolutions, pooling, up-convolution, concat, the
element-wise masks and adds -- runs in the HIP kernels of libsp3d.

Architecture (the paper's Sec. 3 network in the shape the workload list fixes): encoder levels with
channels `channels`, `convs` 3x3x3 conv + ReLU per level (two in the workload list, four in the paper's
own blocks), 2x2x2 max-pool between levels; the last level is the bottleneck; decoder levels mirror the
encoder: 2x2x2 stride-2 transposed conv halving the channels, concat (skip, up), `convs` 3x3x3 conv +
ReLU; a final 1x1x1 conv to `classes`.  Biases are
zero and not passed.  Every 3x3x3 conv input is halo-exchanged first (sp_halo_exchange: pack, delivery and unpack in one pass).

With `halo` = 2 the tensors carry margins that wide and two consecutive layers of a block share
one exchange (the overlap idea of the paper's Sec. 1 applied to a short stack): the first layer of such a group
also computes the voxels around the tile that the later ones read (`grow`), and the backward pass does the same
with the gradients.  The results are bit for bit those of `halo` = 1.

With `flat` the same network is the paper's 2-D U-Net (Sec. 3: same architecture, 2-D convolutions and
poolings, trained on 512 x 512 x 5 slabs): D is a stack of independent slices, the kernels are 3x3 and the
windows 1x2x2, and only H and W halve from level to level.
"""
import numpy as np
import torch

from . import sp3d


LETTERS = "abcdefgh"


def layer_plan(channels=(32, 64, 128, 256), in_ch=1, classes=3, convs=2, flat=False):
    """Names and shapes of all weight tensors, in forward order (flat: the 2-D variant's 3x3 / 2x2 / 1x1)."""
    nd = 2 if flat else 3
    plan = []
    prev = in_ch
    for i, c in enumerate(channels):
        for k in range(convs):
            plan.append(("enc%d_%s" % (i, LETTERS[k]), (3,) * nd + (prev if k == 0 else c, c)))
        prev = c
    for i in range(len(channels) - 2, -1, -1):
        c = channels[i]
        plan.append(("up%d" % i, (2,) * nd + (prev, c)))
        for k in range(convs):
            plan.append(("dec%d_%s" % (i, LETTERS[k]), (3,) * nd + (2 * c if k == 0 else c, c)))
        prev = c
    plan.append(("head", (1,) * nd + (prev, classes)))
    return plan


class UNet:
    def __init__(self, n, dhw, grid, weights, channels=(32, 64, 128, 256), in_ch=1, classes=3,
                 dt=sp3d.SP_BF16, convs=2, halo=1, flat=False, gather=False, grids=None, bits=False):
        self.channels, self.in_ch, self.classes, self.dt = tuple(channels), in_ch, classes, dt
        self.convs = convs
        # Runs of more than two layers would need ReLU masks further around the tiles in the backward pass than
        # the forward pass produces (layer j of a run needs its input's mask j voxels out, the forward pass
        # leaves it run length - j voxels out).
        assert 1 <= halo <= 2
        self.halo = halo
        # gather: layers whose kernels can do it read their margins from the neighbour tiles' interiors
        # (SP_HALO_GATHER) instead of having them exchanged first; the others exchange as before
        self.gather = bool(gather) and halo == 1
        # bits: a layer whose output is the next layer's input also writes the one-bit form of its ReLU mask,
        # and that layer's data gradient reads the bits instead of the activation (where both kernels can)
        self.bits = bool(bits) and halo == 1
        self.free = {}                        # (padded shape, channels) -> released gradient buffers
        self.L = len(channels)
        self.flat = bool(flat)
        # grids: one tile grid per level (default: `grid` everywhere).  The paper allows one or more patches per
        # device (Fig. 1a), and a deep network's coarse levels are small: merging their tiles into fewer, larger
        # ones gives the convolutions longer marches and fuller patches.  Where two neighbouring levels differ, the
        # tensor that crosses (pooled activation, up-convolution input, their gradients) is reassembled and cut
        # again (sp_unpartition + sp_partition on a tensor an eighth of the finer level's size).
        self.grids = [tuple(grid)] * self.L if grids is None else [tuple(q) for q in grids]
        assert len(self.grids) == self.L
        self.g = [sp3d.Geom(n, (dhw[0] if flat else dhw[0] >> i, dhw[1] >> i, dhw[2] >> i), self.grids[i], halo, 0, flat)
                  for i in range(self.L)]
        self.vols = {}                        # (shape) -> volume used to carry a tensor from one grid to another
        for g in self.g:
            assert sp3d.sp_check_geom(g) == sp3d.SP_OK
        self.w = weights                      # name -> device tensor
        self.ws_cache = {}
        self.pool = {}                        # name -> padded tensor, allocated (zeroed) once and reused

    def _buf(self, name, g, c):
        """Padded tensor owned by `name`.  It is zeroed only when first allocated: later steps overwrite the
        interiors, and margins are either rewritten by the halo exchange before anything reads them or
        never read (pooling, up-convolution, 1x1x1 convolution and the element-wise ops use interiors or
        pass margins through)."""
        key = (name, g.padded_shape, c)
        t = self.pool.get(key)
        if t is None:
            t = sp3d.alloc_padded(g, c, self.dt)
            self.pool[key] = t
        return t

    # ---- small helpers -------------------------------------------------------------------------
    def _ws(self, op, g, cin, cout):
        nbytes = sp3d.sp_workspace_bytes(op, g, cin, cout, self.dt)
        key = max(nbytes, 16)
        cur = self.ws_cache.get("buf")
        if cur is None or cur.numel() < key:
            cur = sp3d.alloc_ws(key)
            self.ws_cache["buf"] = cur
        return cur

    def _two_tensor(self, c):
        """the two-tensor convolution entry points need bf16 and channel counts in multiples of 32"""
        return self.dt == sp3d.SP_BF16 and c % 32 == 0

    def _can_grow(self, cin, cout):
        """kernels that compute a grown box: the matrix-core ones (bf16, channels in multiples of 32) and the
        generic fp32 one"""
        return self.dt != sp3d.SP_BF16 or (cin % 32 == 0 and cout % 32 == 0)

    def _groups(self, cin, c):
        """Split the block's layers into runs that share one exchange: [(first layer, number of layers)]."""
        out, k = [], 0
        while k < self.convs:
            s = min(self.halo, self.convs - k) if self._can_grow(cin if k == 0 else c, c) and self._can_grow(c, c) else 1
            out.append((k, s))
            k += s
        return out

    def _plan(self, cin, c):
        """per layer: (exchange before the forward pass, forward grow, position j in its group, group size)"""
        plan = {}
        for k0, s in self._groups(cin, c):
            for j in range(s):
                plan[k0 + j] = (j == 0, s - 1 - j, j, s)
        return plan

    def _gathers(self, op, g, cin, cout):
        return self.gather and sp3d.sp_gather_supported(op, g, cin, cout, self.dt)

    def _x_gathered(self, g, cin, cout):
        """a layer's saved input stays without halos only if both kernels that read them can gather"""
        return self._gathers(sp3d.SP_OP_FWD, g, cin, cout) and self._gathers(sp3d.SP_OP_WGRAD, g, cin, cout)

    def _exchange(self, P, g, c):
        """All tiles share this GPU's memory, so margins are filled straight from the neighbours' interiors.
        Margins at the volume border are left alone: every padded tensor of the driver is zeroed when it is
        allocated and nothing writes beyond the border afterwards, so they hold their zero padding already."""
        sp3d.sp_halo_exchange(P, g.with_opts(sp3d.SP_HALO_KEEP_ZERO), c, self.dt)

    def _mask_bits(self, name, g, cin, cout, last):
        """Buffer for the one-bit ReLU mask of layer `name`'s output, or None if the mask stays a tensor: the
        layer must feed another layer of its block, and both its forward kernel and that layer's data gradient
        (cout -> cout channels) must take the bit form."""
        if (not self.bits or last or not sp3d.sp_relu_bits_supported(sp3d.SP_OP_FWD, g, cin, cout, self.dt)
                or not sp3d.sp_relu_bits_supported(sp3d.SP_OP_DGRAD, g, cout, cout, self.dt)):
            return None
        key = (name + ".bits", g.padded_shape, cout)
        t = self.pool.get(key)
        if t is None:
            t = self.pool[key] = torch.empty(sp3d.sp_relu_bits_bytes(g, cout) // 2, dtype=torch.int16, device="cuda")
        return t

    def _conv(self, Px, name, g, cin, cout, grow=0, bits=None):
        """Px must hold its halos.  Returns relu(conv(Px)) as padded tiles (written: the interiors and `grow`
        voxels around them); with `bits` the one-bit mask of the result goes there as well."""
        Py = self._buf(name + ".y", g, cout)
        gg = g.grown(grow) if grow else g
        if self._x_gathered(g, cin, cout):
            gg = g.with_opts(sp3d.SP_HALO_GATHER)
        if bits is not None:
            sp3d.conv3d_fwd_bits(Px, self.w[name], None, Py, bits, gg, cin, cout, self.dt, sp3d.SP_FLAG_RELU,
                                 self._ws(sp3d.SP_OP_FWD, gg, cin, cout))
        else:
            sp3d.conv3d_fwd(Px, self.w[name], None, Py, gg, cin, cout, self.dt, sp3d.SP_FLAG_RELU,
                            self._ws(sp3d.SP_OP_FWD, gg, cin, cout))
        return Py

    def _block_fwd(self, block, P, g, cin, c, A, P2=None):
        """`convs` conv + ReLU layers; saves every layer input (with halos) and the block output in A.
        With P2 the block input is concat(P, P2) (cin / 2 channels each), never materialised."""
        plan = self._plan(cin, c)
        for k in range(self.convs):
            name = "%s_%s" % (block, LETTERS[k])
            exch, grow = plan[k][0], plan[k][1]
            mb = self._mask_bits(name, g, cin if k == 0 else c, c, k == self.convs - 1)
            if mb is not None:
                A["%s_%s.xbits" % (block, LETTERS[k + 1])] = mb
            if k == 0 and P2 is not None:
                ca = cin // 2
                gg = g.grown(grow) if grow else g
                if self._x_gathered(g, cin, c):
                    gg = g.with_opts(sp3d.SP_HALO_GATHER)
                else:
                    self._exchange(P, g, ca)
                    self._exchange(P2, g, ca)
                A[name + ".x"] = (P, P2)
                Py = self._buf(name + ".y", g, c)
                if mb is not None:
                    sp3d.conv3d_fwd2_bits(P, ca, P2, ca, self.w[name], None, Py, mb, gg, c, self.dt, sp3d.SP_FLAG_RELU,
                                          self._ws(sp3d.SP_OP_FWD, gg, cin, c))
                else:
                    sp3d.conv3d_fwd2(P, ca, P2, ca, self.w[name], None, Py, gg, c, self.dt, sp3d.SP_FLAG_RELU,
                                     self._ws(sp3d.SP_OP_FWD, gg, cin, c))
                P = Py
                continue
            if exch and not self._x_gathered(g, cin if k == 0 else c, c):
                self._exchange(P, g, cin if k == 0 else c)
            A[name + ".x"] = P
            P = self._conv(P, name, g, cin if k == 0 else c, c, grow, mb)
        A[block + ".y"] = P
        return P

    def _block_bwd(self, block, Pg, g, cin, c, grads, need_dx=True, masked_last=False):
        """backward of a block, last layer first; layer k's output is layer k + 1's input.  masked_last: Pg is
        already d/dz of the last layer (its producer applied the ReLU mask of the block output)."""
        A = self.A
        plan = self._plan(cin, c)
        for k in range(self.convs - 1, -1, -1):
            name = "%s_%s" % (block, LETTERS[k])
            Py = A[block + ".y"] if k == self.convs - 1 else A["%s_%s.x" % (block, LETTERS[k + 1])]
            # Layer k > 0 reads the ReLU output of layer k - 1: its data gradient applies that mask itself.
            # Inside a run of layers that share one exchange only the last layer's d/dz is exchanged; layer j of
            # the run then also produces the j voxels of d/dx around the tile that layer j - 1 reads.
            j, s = plan[k][2], plan[k][3]
            Pg = self._conv_bwd(name, A[name + ".x"], Py, Pg, g, cin if k == 0 else c, c, grads,
                                need_dx=(need_dx or k > 0), masked=(k < self.convs - 1 or masked_last),
                                mask_next=(k > 0),
                                exchange=(j == s - 1), grow=j)
        return Pg

    # gradient buffers are short-lived: they come from a free list keyed by shape and go back to it as
    # soon as their consumer has run, so the backward pass needs a few of the largest tensors, not one per
    # layer
    def _regrid(self, P, g_from, g_to, c, out):
        """The tensor P (tiles of g_from) as tiles of g_to (same volume, another grid), written into `out`."""
        assert (g_from.n, g_from.d, g_from.h, g_from.w) == (g_to.n, g_to.d, g_to.h, g_to.w)
        shape = (g_from.n, g_from.d, g_from.h, g_from.w, c)
        V = self.vols.get(shape)
        if V is None:
            V = self.vols[shape] = torch.empty(shape, dtype=P.dtype, device="cuda")
        sp3d.sp_unpartition(P, V, g_from, c, self.dt)
        sp3d.sp_partition(V, out, g_to, c, self.dt)
        return out

    def _same_grid(self, i, j):
        return self.grids[i] == self.grids[j]

    def _tmp(self, g, c):
        key = (g.padded_shape, c)
        lst = self.free.setdefault(key, [])
        return lst.pop() if lst else sp3d.alloc_padded(g, c, self.dt)

    def _release(self, t, g, c):
        self.free.setdefault((g.padded_shape, c), []).append(t)

    # ---- forward ----------------------------------------------------------------------------------
    def forward(self, x_vol):
        """x_vol: device volume [n,d,h,w,in_ch].  Returns the logits volume; keeps what backward needs."""
        dt, ch = self.dt, self.channels
        A = {}                                   # saved activations (padded, halos exchanged where needed)
        P = self._buf("input", self.g[0], self.in_ch)
        sp3d.sp_partition(x_vol, P, self.g[0], self.in_ch, dt)
        prev = self.in_ch
        for i in range(self.L):
            g, c = self.g[i], ch[i]
            if i > 0:
                Pp = self._buf("pool%d" % i, g, prev)
                if self._same_grid(i - 1, i):
                    sp3d.sp_maxpool2_fwd(P, Pp, self.g[i - 1], prev, dt)
                else:                                # pooled on the finer level's grid, then cut for this level's
                    gq = sp3d.coarse_geom(self.g[i - 1])
                    Pq = self._buf("pool%d.q" % i, gq, prev)
                    sp3d.sp_maxpool2_fwd(P, Pq, self.g[i - 1], prev, dt)
                    self._regrid(Pq, gq, g, prev, Pp)
                P = Pp
            P = self._block_fwd("enc%d" % i, P, g, prev, c, A)   # level output: pool input / skip / ReLU mask
            prev = c
        for i in range(self.L - 2, -1, -1):
            g, c = self.g[i], ch[i]
            if not self._same_grid(i, i + 1):        # the coarse tensor on the finer level's grid
                gq = sp3d.coarse_geom(g)
                P = self._regrid(P, self.g[i + 1], gq, prev, self._buf("up%d.q" % i, gq, prev))
            A["up%d.x" % i] = P
            Pu = self._buf("up%d.y" % i, g, c)
            sp3d.sp_upconv2_fwd(P, self.w["up%d" % i], None, Pu, g, prev, c, dt)
            if self._two_tensor(c):                  # convolve concat(skip, up) without building it
                P = self._block_fwd("dec%d" % i, A["enc%d.y" % i], g, 2 * c, c, A, P2=Pu)
            else:
                Pc = self._buf("cat%d" % i, g, 2 * c)
                sp3d.sp_concat(A["enc%d.y" % i], c, Pu, c, Pc, g, dt)
                P = self._block_fwd("dec%d" % i, Pc, g, 2 * c, c, A)
            prev = c
        A["head.x"] = P
        Pl = self._buf("logits", self.g[0], self.classes)
        sp3d.sp_pointwise_fwd(P, self.w["head"], None, Pl, self.g[0], prev, self.classes, dt)
        self.A = A
        g0 = self.g[0]
        out = torch.empty((g0.n, g0.d, g0.h, g0.w, self.classes), dtype=Pl.dtype, device="cuda")
        sp3d.sp_unpartition(Pl, out, g0, self.classes, dt)
        return out

    # ---- backward ---------------------------------------------------------------------------------
    def _conv_bwd(self, name, Px, Py, Pdy, g, cin, cout, grads, need_dx=True, masked=False, mask_next=False,
                  exchange=True, grow=0):
        """Backward of y = relu(conv(x)): Pdy is d/dy (interiors valid), or already d/dz if `masked`.
        Returns d/dx (padded); with `mask_next` (x is itself a ReLU output) the ReLU mask of x is applied
        in the same pass, so the result is the previous layer's d/dz."""
        dt = self.dt
        if not masked:
            sp3d.sp_relu_bwd(Pdy, Py, Pdy, g, cout, dt)               # dz in place
        dw = torch.empty(tuple(self.w[name].shape), dtype=torch.float32, device="cuda")
        if isinstance(Px, tuple):                 # x = concat(Px[0], Px[1]): gradients go to two tensors
            ca = cin // 2
            gx = g.with_opts(sp3d.SP_HALO_GATHER) if self._x_gathered(g, cin, cout) else g
            sp3d.conv3d_wgrad2(Px[0], ca, Px[1], ca, Pdy, dw, None, gx, cout, dt,
                               self._ws(sp3d.SP_OP_WGRAD, g, cin, cout))
            grads[name] = dw
            gz = g
            if self._gathers(sp3d.SP_OP_DGRAD, g, cin, cout):
                gz = g.with_opts(sp3d.SP_HALO_GATHER)
            elif exchange:
                self._exchange(Pdy, g, cout)
            Pa, Pb = self._tmp(g, ca), self._tmp(g, ca)
            sp3d.conv3d_dgrad2(Pdy, self.w[name], Pa, ca, Pb, ca, gz, cout, dt,
                               self._ws(sp3d.SP_OP_DGRAD, g, cin, cout))          # first layer of its run: no grow
            self._release(Pdy, g, cout)
            return (Pa, Pb)
        gx = g.with_opts(sp3d.SP_HALO_GATHER) if self._x_gathered(g, cin, cout) else g
        sp3d.conv3d_wgrad(Px, Pdy, dw, None, gx, cin, cout, dt, self._ws(sp3d.SP_OP_WGRAD, g, cin, cout))
        grads[name] = dw
        Pdx = None
        if need_dx:
            gg = g.grown(grow) if grow else g
            if self._gathers(sp3d.SP_OP_DGRAD, g, cin, cout):
                gg = g.with_opts(sp3d.SP_HALO_GATHER)
            elif exchange:
                self._exchange(Pdy, g, cout)
            Pdx = self._tmp(g, cin)
            xbits = self.A.get(name + ".xbits") if mask_next else None
            if xbits is not None:
                sp3d.conv3d_dgrad_bits(Pdy, self.w[name], xbits, Pdx, gg, cin, cout, dt,
                                       self._ws(sp3d.SP_OP_DGRAD, gg, cin, cout))
            elif mask_next:
                sp3d.conv3d_dgrad_relu(Pdy, self.w[name], Px, Pdx, gg, cin, cout, dt,
                                       self._ws(sp3d.SP_OP_DGRAD, gg, cin, cout))
            else:
                sp3d.conv3d_dgrad(Pdy, self.w[name], Pdx, gg, cin, cout, dt,
                                  self._ws(sp3d.SP_OP_DGRAD, gg, cin, cout))
        self._release(Pdy, g, cout)
        return Pdx

    def loss(self, labels_vol, w_dice=0.9, w_ce=0.1, eps=1.0):
        """Soft Dice + cross-entropy of the logits of the last forward() against labels_vol (device volume
        [n,d,h,w,1] of the tensor dtype holding class indices).  Returns a 1-element device tensor and leaves
        d loss / d logits in the padded gradient buffer that backward(None) starts from."""
        g0, dt = self.g[0], self.dt
        Pl = self._buf("logits", g0, self.classes)
        Plab = self._buf("labels", g0, 1)
        sp3d.sp_partition(labels_vol, Plab, g0, 1, dt)
        Pd = self._buf("dlogits", g0, self.classes)
        out = torch.empty(1, dtype=torch.float32, device="cuda")
        nbytes = sp3d.sp_workspace_bytes(sp3d.SP_OP_LOSS, g0, self.classes, 1, dt)
        cur = self.ws_cache.get("buf")
        if cur is None or cur.numel() < nbytes:
            cur = sp3d.alloc_ws(nbytes)
            self.ws_cache["buf"] = cur
        sp3d.sp_dice_ce_loss(Pl, Plab, Pd, out, None, g0, self.classes, dt, w_dice, w_ce, eps, cur)
        return out

    def backward(self, dlogits_vol, input_grad=True):
        """dlogits_vol: device volume [n,d,h,w,classes], or None to start from the gradient loss() left.
        Returns (grads by layer name, dx volume or None)."""
        dt, ch, A = self.dt, self.channels, self.A
        grads = {}
        g0 = self.g[0]
        Pd = self._buf("dlogits", g0, self.classes)
        if dlogits_vol is not None:
            sp3d.sp_partition(dlogits_vol, Pd, g0, self.classes, dt)
        c0 = ch[0]
        dp = torch.empty(tuple(self.w["head"].shape), dtype=torch.float32, device="cuda")
        Pg = self._tmp(g0, c0)
        # the head reads the ReLU output of the last decoder block: its data gradient applies that mask, in the
        # same sweep over that activation as the weight gradient
        sp3d.sp_pointwise_bwd_relu(A["head.x"], Pd, self.w["head"], Pg, dp, None, g0, c0, self.classes, dt,
                                   self._ws(sp3d.SP_OP_POINTWISE_WGRAD, g0, c0, self.classes))
        grads["head"] = dp
        skip_grad = {}
        for i in range(0, self.L - 1):
            g, c = self.g[i], ch[i]
            up_in = ch[i + 1]
            Pg = self._block_bwd("dec%d" % i, Pg, g, 2 * c, c, grads, masked_last=(i == 0))   # -> d concat(skip, up)
            if isinstance(Pg, tuple):
                Ps, Pu = Pg
            else:
                Ps, Pu = self._tmp(g, c), self._tmp(g, c)
                sp3d.sp_split(Pg, Ps, c, Pu, c, g, dt)
                self._release(Pg, g, 2 * c)
            skip_grad[i] = Ps
            du = torch.empty(tuple(self.w["up%d" % i].shape), dtype=torch.float32, device="cuda")
            sp3d.sp_upconv2_wgrad(A["up%d.x" % i], Pu, du, None, g, up_in, c, dt,
                                  self._ws(sp3d.SP_OP_UPCONV_WGRAD, g, up_in, c))
            grads["up%d" % i] = du
            if self._same_grid(i, i + 1):
                Pg = self._tmp(self.g[i + 1], up_in)
                sp3d.sp_upconv2_dgrad(Pu, self.w["up%d" % i], Pg, g, up_in, c, dt)
            else:
                gq = sp3d.coarse_geom(g)
                Pq = self._tmp(gq, up_in)
                sp3d.sp_upconv2_dgrad(Pu, self.w["up%d" % i], Pq, g, up_in, c, dt)
                Pg = self._regrid(Pq, gq, self.g[i + 1], up_in, self._tmp(self.g[i + 1], up_in))
                self._release(Pq, gq, up_in)
            self._release(Pu, g, c)
        joined = False            # Pg already is d/dz of the level's last layer (pool backward + skip + ReLU mask)
        for i in range(self.L - 1, -1, -1):
            g, c = self.g[i], ch[i]
            cin = self.in_ch if i == 0 else ch[i - 1]
            Pg = self._block_bwd("enc%d" % i, Pg, g, cin, c, grads, need_dx=(i > 0 or input_grad), masked_last=joined)
            if i > 0:
                # the level above: gradient through its pooling, plus the one that came through its skip
                # connection, masked by the ReLU of its output (which is the pooling input), in one sweep
                Ps = skip_grad.pop(i - 1)
                if not self._same_grid(i - 1, i):     # the pooled tensor's gradient on the finer level's grid
                    gq = sp3d.coarse_geom(self.g[i - 1])
                    Pq = self._regrid(Pg, g, gq, cin, self._tmp(gq, cin))
                    self._release(Pg, g, cin)
                    Pg, g = Pq, gq
                sp3d.sp_maxpool2_bwd_join(A["enc%d.y" % (i - 1)], Pg, Ps, Ps, self.g[i - 1], cin, dt)
                self._release(Pg, g, cin)
                Pg, joined = Ps, True
        dx = None
        if input_grad:
            dx = torch.empty((g0.n, g0.d, g0.h, g0.w, self.in_ch), dtype=Pg.dtype, device="cuda")
            sp3d.sp_unpartition(Pg, dx, g0, self.in_ch, dt)
            self._release(Pg, g0, self.in_ch)
        return grads, dx
