"""The U-Net data flow replayed layer by layer through the library's layer entry points, with
every layer's output checked against the oracle applied to the GPU's OWN inputs of that layer
(teacher forcing).

Why: two bf16 realisations of a deep net legitimately drift apart (a one-ulp difference in a
stored activation flips a ReLU mask or a pooling arg-max at a near-tie, and each flip changes a
gradient element by its full size), so an end-to-end gradient cannot be held to the per-layer
tolerance.  Instead (a) each layer is held to it given identical inputs, and (b) the whole-network
entry point must reproduce this chain bit for bit (same kernels, same order).

verify=True checks every layer in full (small volumes).  verify="sampled" is for full-size volumes:
the 3x3x3 convolutions (forward, data gradient, weight gradient) are checked on sampled outputs
the oracle computes one by one from the GPU's own inputs of that layer -- all channels of a few
hundred voxels that include the corners and both sides of tile boundaries -- while every O(V) op
(statistics, normalise+ReLU and its backward, pooling, the transposed convolution, the head) is
still checked in full, sample by sample of the batch.
"""
import numpy as np
import torch

import oracle as O
from gpu_util import DEV, as64, check

F32 = torch.float32


class Chain:
    def __init__(self, L, levels, base, in_ch, classes, affine, dtype, names, params, eps=1e-5, verify=True):
        self.L, self.levels, self.base, self.in_ch, self.K = L, levels, base, in_ch, classes
        self.affine, self.dtype, self.eps, self.verify = affine, dtype, eps, verify
        self.P = dict(zip(names, params))
        self.names = names
        self.worst = {}
        self.sampled = verify == "sampled"
        self.full = verify is True
        self.rng = np.random.Generator(np.random.PCG64(77))
        self.nsample = 384
        self.checked = {}

    # ---- sampled verification ---------------------------------------------------------------
    def _coords(self, shape, nsample=None):
        """Voxels (n,d,h,w): all corners, both sides of the 8- and 16-voxel tile boundaries along
        each axis, then uniform random ones."""
        N, D, H, W = shape
        nsample = self.nsample if nsample is None else nsample
        pts = set()
        for n in {0, N - 1}:
            for d in {0, D - 1}:
                for h in {0, H - 1}:
                    for w in {0, W - 1}:
                        pts.add((n, d, h, w))
        for a in (3, 4, 7, 8, 15, 16, 31, 32, 63, 64):
            if a < min(D, H, W):
                pts.add((N - 1, a, a, a))
                pts.add((0, a, 0, W - 1 - a))
                pts.add((0, D - 1, a, 0))
                pts.add((N - 1, 0, H - 1 - a, a))
        total = N * D * H * W
        while len(pts) < min(nsample, total):
            pts.add((int(self.rng.integers(N)), int(self.rng.integers(D)), int(self.rng.integers(H)), int(self.rng.integers(W))))
        return sorted(pts)

    @staticmethod
    def _host(t):
        return t.detach().cpu().float().numpy()

    def _count(self, what):
        self.checked[what] = self.checked.get(what, 0) + 1

    def _sampled_conv(self, kind, name, a, w, out):
        """kind 'fwd': out = conv(a, w); 'dgrad': out = conv^T(a, w)."""
        # the oracle spends 27 * Ci * Co multiply-adds per sampled voxel: fewer voxels for very wide layers
        per_voxel = 27 * int(w.shape[0]) * int(w.shape[4])
        coords = self._coords(out.shape[:4], max(128, min(self.nsample, int(3e9 // per_voxel))))
        ah, oh = self._host(a), self._host(out)
        f = O.conv3d_fwd_at if kind == "fwd" else O.conv3d_dgrad_at
        ref = f(ah, as64(w), None, coords) if kind == "fwd" else f(ah, as64(w), coords)
        got = np.stack([oh[c] for c in coords]).astype(np.float64)
        e = check(got, ref, self.dtype, f"conv {kind} (sampled): {name}")
        self.worst[f"conv {kind}"] = max(self.worst.get(f"conv {kind}", 0.0), e)
        self._count(f"conv {kind}")

    @staticmethod
    def _block_edges(C):
        """Channel indices on both sides of every 32-channel block boundary (the matrix-core kernels' workgroup and
        fragment blocks), plus the ends."""
        e = {0, C - 1}
        for b in range(32, C, 32):
            e.update((b - 1, b))
        return sorted(e)

    def _wgrad_entries(self, Co, Ci, per_tap=10):
        """>= 27 * per_tap entries (co, kd, kh, kw, ci): every one of the 27 taps, and across the taps every
        32-channel block boundary of both channel axes (cycled through, so wide layers are covered too), then
        random ones."""
        eo, ei = self._block_edges(Co), self._block_edges(Ci)
        # at most 10 distinct channels per axis (the oracle gathers one plane of the volume per channel): the two
        # ends and a seeded choice of the block boundaries
        pick = lambda e: sorted({e[0], e[-1], *[e[int(i)] for i in self.rng.choice(len(e), size=min(8, len(e)), replace=False)]})
        eo, ei = pick(eo), pick(ei)
        ro = [int(v) for v in self.rng.integers(Co, size=4)]
        ri = [int(v) for v in self.rng.integers(Ci, size=4)]
        ent = set()
        io = ii = 0
        for t in range(27):
            kd, kh, kw = t // 9, (t // 3) % 3, t % 3
            for j in range(per_tap):
                if j < per_tap // 2:      # boundary x boundary
                    co, ci = eo[io % len(eo)], ei[ii % len(ei)]
                    io += 1
                    ii += 3               # a different stride, so the pairs do not stay in step
                elif j < per_tap - 2:     # boundary x random, random x boundary
                    if j % 2:
                        co, ci = eo[io % len(eo)], ri[int(self.rng.integers(4))]
                        io += 1
                    else:
                        co, ci = ro[int(self.rng.integers(4))], ei[ii % len(ei)]
                        ii += 1
                else:
                    co, ci = ro[int(self.rng.integers(4))], ri[int(self.rng.integers(4))]
                ent.add((co, kd, kh, kw, ci))
        allc, alli = eo + ro, ei + ri
        while len(ent) < min(256, 27 * len(set(allc)) * len(set(alli))):   # duplicates of a narrow layer: top up
            ent.add((allc[int(self.rng.integers(len(allc)))], int(self.rng.integers(3)), int(self.rng.integers(3)),
                     int(self.rng.integers(3)), alli[int(self.rng.integers(len(alli)))]))
        return sorted(ent)

    def _sampled_wgrad(self, name, x, dz, dw):
        Co, _, _, _, Ci = dw.shape
        ent = self._wgrad_entries(Co, Ci) if Ci * Co * 27 >= 270 else [(co, t // 9, (t // 3) % 3, t % 3, ci)
                                                                        for co in range(Co) for t in range(27) for ci in range(Ci)]
        ref = O.conv3d_wgrad_at(self._host(x), self._host(dz), ent)
        dwh = as64(dw)
        got = np.array([dwh[e] for e in ent])
        # scale: the largest entry of the whole gradient tensor (the metric of the full check)
        err = float(np.max(np.abs(got - ref)) / np.max(np.abs(dwh)))
        tol = 2e-3 if self.dtype != F32 else 1e-4
        assert err <= tol, f"conv wgrad (sampled, {len(ent)} entries): {name}: E_inf = {err:.2e} > {tol:g}"
        self.worst["conv wgrad"] = max(self.worst.get("conv wgrad", 0.0), err)
        self._count("conv wgrad")

    def _per_sample(self, what, fn, *tensors, outs, ignore_fn=None, tol=None, dtype=None):
        """Full check of an O(V) op, one batch sample at a time: fn(*float64 slices) -> reference
        arrays matching `outs`."""
        N = tensors[0].shape[0]
        for n in range(N):
            refs = fn(*[as64(t[n:n + 1]) for t in tensors])
            if not isinstance(refs, (tuple, list)):
                refs = (refs,)
            for o, r in zip(outs, refs):
                ig = ignore_fn(n) if ignore_fn is not None else None
                e = check(as64(o[n:n + 1]), r, dtype or self.dtype, what, ignore=ig, tol=tol)
                key = what.split(":")[0]
                self.worst[key] = max(self.worst.get(key, 0.0), e)
        self._count(what.split(":")[0])

    def _chk(self, gpu, ref, what, ignore=None, tol=None):
        if self.verify:
            e = check(as64(gpu), ref, self.dtype, what, ignore=ignore, tol=tol)
            self.worst[what.split(":")[0]] = max(self.worst.get(what.split(":")[0], 0.0), e)

    def chan(self, l):
        return self.base << (l - 1)

    # ---- forward ------------------------------------------------------------------------------
    def conv_in_relu(self, name, x, y_out=None):
        L, P = self.L, self.P
        w = P[name + ".w"]
        g, b = P.get(name + ".gamma"), P.get(name + ".beta")
        N, D, H, W, _ = x.shape
        Co = w.shape[0]
        z = torch.empty((N, D, H, W, Co), dtype=self.dtype, device=DEV)
        st = torch.empty((N, Co, 2), dtype=F32, device=DEV)
        L.lamp_conv3d_fwd(x, w, z, stats_out=st, eps=self.eps)
        y = y_out if y_out is not None else torch.empty_like(z)
        L.lamp_inorm_relu(z, y, st, gamma=g, beta=b, eps=self.eps, stats_given=True)
        if self.sampled:
            self._sampled_conv("fwd", name, x, w, z)
            g64 = None if g is None else as64(g)
            b64 = None if b is None else as64(b)
            for n in range(N):
                y_ref, st_ref = O.inorm_relu(as64(z[n:n + 1]), g64, b64, self.eps)
                e = check(as64(y[n:n + 1]), y_ref, self.dtype, f"inorm+relu: {name}")
                self.worst["inorm+relu"] = max(self.worst.get("inorm+relu", 0.0), e)
                s_gpu = as64(st[n:n + 1])
                np.testing.assert_allclose(s_gpu[..., 0], st_ref[..., 0], atol=1e-4 * max(1.0, np.abs(st_ref[..., 0]).max()))
                np.testing.assert_allclose(s_gpu[..., 1], st_ref[..., 1], rtol=2e-4)
            self._count("inorm+relu")
        if self.full:
            self._chk(z, O.conv3d_fwd(as64(x), as64(w)), f"conv fwd: {name}")
            y_ref, st_ref = O.inorm_relu(as64(z), None if g is None else as64(g), None if b is None else as64(b), self.eps)
            self._chk(y, y_ref, f"inorm+relu: {name}")
            np.testing.assert_allclose(as64(st)[..., 0], st_ref[..., 0], atol=1e-4 * max(1.0, np.abs(st_ref[..., 0]).max()))
            np.testing.assert_allclose(as64(st)[..., 1], st_ref[..., 1], rtol=2e-4)
        return dict(x=x, z=z, st=st, y=y, name=name)

    def block(self, prefix, x, y2_out=None):
        c1 = self.conv_in_relu(prefix + ".conv1", x)
        c2 = self.conv_in_relu(prefix + ".conv2", c1["y"], y2_out)
        return c1, c2

    def forward(self, x):
        L, Lv = self.L, self.levels
        N = x.shape[0]
        self.enc, self.dec, self.cat, self.pooled = {}, {}, {}, {}
        cur = x
        for l in range(1, Lv + 1):
            C = self.chan(l)
            y2 = None
            if l < Lv:
                _, D, H, W, _ = cur.shape
                self.cat[l] = torch.zeros((N, D, H, W, 2 * C), dtype=self.dtype, device=DEV)
                y2 = self.cat[l][..., :C]
            self.enc[l] = self.block(f"enc{l}", cur, y2)
            if l < Lv:
                yv = self.enc[l][1]["y"]
                p = torch.empty((N, yv.shape[1] // 2, yv.shape[2] // 2, yv.shape[3] // 2, C), dtype=self.dtype, device=DEV)
                L.lamp_maxpool2_fwd(yv, p)
                if self.verify:
                    for n in range(N):
                        np.testing.assert_array_equal(as64(p[n:n + 1]), O.maxpool2_fwd(as64(yv[n:n + 1])))
                    self._count("pool fwd")
                self.pooled[l] = p
                cur = p
        cur = self.enc[Lv][1]["y"]
        for l in range(Lv - 1, 0, -1):
            C = self.chan(l)
            up = self.cat[l][..., C:]
            wt, bt = self.P[f"dec{l}.up.w"], self.P[f"dec{l}.up.b"]
            L.lamp_convtr3d(cur, wt, up, bias=bt)
            if self.full:
                self._chk(up, O.convtr3d_fwd(as64(cur), as64(wt), as64(bt)), f"convtr fwd: dec{l}")
            if self.sampled:
                self._per_sample(f"convtr fwd: dec{l}", lambda a: O.convtr3d_fwd(a, as64(wt), as64(bt)), cur, outs=(up,))
            self.dec[l] = self.block(f"dec{l}", self.cat[l])
            self.dec[l] = self.dec[l] + (cur,)
            cur = self.dec[l][1]["y"]
        self.top = cur
        logits = torch.empty(tuple(cur.shape[:4]) + (self.K,), dtype=F32, device=DEV)
        L.lamp_head_fwd(cur, self.P["head.w"], self.P["head.b"], logits)
        if self.sampled:
            self._per_sample("head fwd", lambda a: O.head_fwd(a, as64(self.P["head.w"]), as64(self.P["head.b"])),
                             cur, outs=(logits,), tol=1e-5, dtype=F32)
        if self.full:
            check(as64(logits), O.head_fwd(as64(cur), as64(self.P["head.w"]), as64(self.P["head.b"])), F32, "head fwd", tol=1e-5)
        return logits

    # ---- backward -----------------------------------------------------------------------------
    def _inorm_bwd(self, c, g, grads, run):
        """The InstanceNorm + ReLU backward of conv unit c: run(dz_out, dgamma, dbeta) launches the library call that
        turns the gradient g w.r.t. c['y'] into dz (written to dz_out, which may be g) -- the stand-alone call, or the
        call fused with the data gradient that produced g; the result is checked against the oracle's backward of g."""
        P, name = self.P, c["name"]
        gm, bt = P.get(name + ".gamma"), P.get(name + ".beta")
        dg = torch.empty_like(gm) if gm is not None else None
        db = torch.empty_like(bt) if bt is not None else None
        g_in = as64(g) if self.full else None
        g_dev = g.clone() if self.sampled else None
        g = run(g, dg, db)
        if self.sampled:
            g64 = None if gm is None else as64(gm)
            b64 = None if bt is None else as64(bt)
            dg_ref = db_ref = 0.0
            for n in range(g.shape[0]):
                zn = as64(c["z"][n:n + 1])
                dz_ref, dgn, dbn = O.inorm_relu_bwd(as64(g_dev[n:n + 1]), zn, g64, b64, self.eps)
                u_ref, _ = O.inorm_relu(zn, g64, b64, self.eps, relu=False)
                e = check(as64(g[n:n + 1]), dz_ref, self.dtype, f"inorm bwd: {name}", ignore=np.abs(u_ref) <= 1e-3)
                self.worst["inorm bwd"] = max(self.worst.get("inorm bwd", 0.0), e)
                dg_ref, db_ref = dg_ref + dgn, db_ref + dbn
            if gm is not None:
                check(as64(dg), dg_ref, F32, f"dgamma: {name}", tol=2e-3)
                check(as64(db), db_ref, F32, f"dbeta: {name}", tol=2e-3)
            self._count("inorm bwd")
            del g_dev
        if self.full:
            g64 = None if gm is None else as64(gm)
            b64 = None if bt is None else as64(bt)
            dz_ref, dg_ref, db_ref = O.inorm_relu_bwd(g_in, as64(c["z"]), g64, b64, self.eps)
            u_ref, _ = O.inorm_relu(as64(c["z"]), g64, b64, self.eps, relu=False)
            near = np.abs(u_ref) <= 1e-3
            self._chk(g, dz_ref, f"inorm bwd: {name}", ignore=near)
        if gm is not None:
            grads[name + ".gamma"], grads[name + ".beta"] = dg, db
        return g

    def conv_bwd(self, c, g, grads, want_dx, dx_out=None, below=None, dz_ready=False):
        """g: gradient w.r.t. c['y'] (overwritten with dz; dz_ready: g already is dz).  Returns dx (or None).
        below: the conv unit whose activated output is this conv's input -- the data gradient and that unit's
        InstanceNorm + ReLU backward then run as the one fused library call, as in the network entry points, and what
        is returned is the gradient w.r.t. that unit's z (pass it on with dz_ready=True)."""
        L, P, name = self.L, self.P, c["name"]
        w = P[name + ".w"]
        if not dz_ready:
            gm, bt = P.get(name + ".gamma"), P.get(name + ".beta")

            def run(gbuf, dg, db):
                L.lamp_inorm_relu_bwd(gbuf, c["z"], c["st"], gbuf, gamma=gm, beta=bt, dgamma=dg, dbeta=db)
                return gbuf
            g = self._inorm_bwd(c, g, grads, run)
        dw = torch.empty(w.shape, dtype=F32, device=DEV)
        L.lamp_conv3d_wgrad(c["x"], g, dw)
        if self.sampled:
            self._sampled_wgrad(name, c["x"], g, dw)
        if self.full:
            self._chk(dw, O.conv3d_wgrad(as64(c["x"]), as64(g))[0], f"conv wgrad: {name}",
                      tol=2e-3 if self.dtype != F32 else 1e-4)
        grads[name + ".w"] = dw
        if not want_dx:
            return None
        dx = dx_out if dx_out is not None else torch.empty_like(c["x"])
        if below is None:
            L.lamp_conv3d_dgrad(g, w, dx)
        else:
            # data gradient into dx, the backward of the unit below into a buffer of its own, so that both can be
            # checked (the network runs the same call in place: the same bits, the backward being element-wise)
            assert dx_out is None
            gmb, btb = P.get(below["name"] + ".gamma"), P.get(below["name"] + ".beta")
            dzb = torch.empty_like(dx)

            def run_fused(gbuf, dg, db):
                L.lamp_conv3d_dgrad_inorm_relu_bwd(g, w, dx, below["z"], below["st"], dzb, gamma=gmb, beta=btb, dgamma=dg, dbeta=db)
                return dzb
            # the stand-alone data gradient first: it gives the backward's input for the checks below, and the fused
            # call, launched by _inorm_bwd, must write the same bits over it
            L.lamp_conv3d_dgrad(g, w, dx)
        if self.sampled:
            self._sampled_conv("dgrad", name, g, w, dx)
        if self.full:
            self._chk(dx, O.conv3d_dgrad(as64(g), as64(w)), f"conv dgrad: {name}")
        if below is None:
            return dx
        dx_alone = dx.clone()
        out = self._inorm_bwd(below, dx, grads, run_fused)
        assert torch.equal(dx, dx_alone), "the fused call's data gradient differs from lamp_conv3d_dgrad"
        return out

    def backward(self, labels):
        L, Lv = self.L, self.levels
        grads = {}
        loss = torch.empty((), dtype=F32, device=DEV)
        top = self.top
        g = torch.empty(top.shape, dtype=self.dtype, device=DEV)
        dwh = torch.empty(self.P["head.w"].shape, dtype=F32, device=DEV)
        dbh = torch.empty(self.P["head.b"].shape, dtype=F32, device=DEV)
        logits = torch.empty(tuple(top.shape[:4]) + (self.K,), dtype=F32, device=DEV)
        L.lamp_head_ce(top, self.P["head.w"], self.P["head.b"], labels, loss, logits=logits, dx=g, dwh=dwh, dbh=dbh)
        if self.verify:  # O(V * C * K): in full at any size
            loss_ref, dl = O.cross_entropy(as64(logits), labels.cpu().numpy())
            assert abs(loss.item() - loss_ref) <= 1e-5 * max(1.0, abs(loss_ref))
            gy, gw, gb = O.head_bwd(as64(top), as64(self.P["head.w"]), dl)
            self._chk(g, gy, "head dx")
            self._chk(dwh, gw, "head dW", tol=1e-4)
            self._chk(dbh, gb, "head db", tol=1e-4)
        grads["head.w"], grads["head.b"] = dwh, dbh
        skip_g = {}
        for l in range(1, Lv):
            C = self.chan(l)
            c1, c2, upx = self.dec[l]
            g = self.conv_bwd(c2, g, grads, True, below=c1)
            gcat = torch.empty_like(self.cat[l])
            self.conv_bwd(c1, g, grads, True, dx_out=gcat, dz_ready=True)
            skip_g[l] = gcat[..., :C]
            gup = gcat[..., C:]
            wt = self.P[f"dec{l}.up.w"]
            g = torch.empty_like(upx)
            dwt = torch.empty(wt.shape, dtype=F32, device=DEV)
            dbt = torch.empty((C,), dtype=F32, device=DEV)
            L.lamp_convtr3d_bwd(upx, wt, gup, dx=g, dwt=dwt, dbias=dbt)
            if self.verify:  # O(V * C^2): in full at any size
                dx_ref, dwt_ref, db_ref = O.convtr3d_bwd(as64(upx), as64(wt), as64(gup))
                self._chk(g, dx_ref, f"convtr dgrad: dec{l}")
                self._chk(dwt, dwt_ref, f"convtr wgrad: dec{l}", tol=2e-3 if self.dtype != F32 else 1e-4)
                self._chk(dbt, db_ref, f"convtr dbias: dec{l}", tol=1e-4)
            grads[f"dec{l}.up.w"], grads[f"dec{l}.up.b"] = dwt, dbt
        for l in range(Lv, 0, -1):
            c1, c2 = self.enc[l]
            if l < Lv:
                gy = torch.empty(c2["y"].shape, dtype=self.dtype, device=DEV)
                L.lamp_maxpool2_bwd(c2["y"], g, gy, add=skip_g[l])
                if self.sampled:
                    sk = skip_g[l]
                    self._per_sample(f"pool bwd: enc{l}", lambda a, b, c_: O.maxpool2_bwd(a, b) + c_, c2["y"], g, sk,
                                     outs=(gy,), tol=4e-3 if self.dtype != F32 else 1e-6)
                if self.full:
                    ref = O.maxpool2_bwd(as64(c2["y"]), as64(g)) + as64(skip_g[l])
                    self._chk(gy, ref, f"pool bwd: enc{l}", tol=4e-3 if self.dtype != F32 else 1e-6)
                g = gy
            g = self.conv_bwd(c2, g, grads, True, below=c1)
            g = self.conv_bwd(c1, g, grads, l > 1, dz_ready=True)
        return loss, grads
