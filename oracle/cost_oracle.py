"""Independent implementation of the published cost function of the fusion-group tuner (TEST
INFRASTRUCTURE ONLY; shares no code with the GPU library).

The cost function is ours, not the paper's: the paper times every candidate on the hardware
(Sec. V "Oracle Case": reduced brute force) and its greedy pass only uses operation count and
channel size (Sec. IV).  Here a group's cost is an integer number of picoseconds computed from
the tiling the library would use (cost model, version 3).  It is
implemented twice, in the library (C++) and here (Python), so that the library's exact tuner can
be checked bit for bit against exhaustive enumeration (plan_oracle.best_plan_exhaustive).

The paper prints no cost function, so nothing here can be pinned against it (parity unpinned): this
module is the second, independent statement of our own definition, and what it checks is that the
library's planner implements exactly that definition and minimises it exactly.

cost(first, last, budget) = min over the candidate tilings of the group of
    (C_LAUNCH + max(compute, memory)) * PS_PER_CYCLE
or None if the layers cannot run as one group / no candidate fits on-chip memory.
"""

# ---- constants of cost model version 3 ----
PS_PER_CYCLE = 465
HBM_BYTES_PER_CYCLE = 3300
CU_BYTES_PER_CYCLE = 12
L2_BYTES_PER_CYCLE = 48
C_LAUNCH = 9000
C_TILE = 6000
C_LAT = 5000
C_STAGE_VEC = 120
C_IM2COL = 150
C_ROWFOLD = 400
C_ROUND = 1500
C_ROUND_VEC = 300
C_BARRIER = 500
C_EPI = 900
C_KSPLIT = 2500
C_VALU = 100
C_STAGE = 1200
C_STORE_VEC = 80
C_STORE = 1600
MFMA_CYCLES = 32
FC_BYTES_PER_CYCLE = 1400
FC_SPLIT_HBM_BYTES_PER_CYCLE = 1900
GAP_BYTES_PER_CYCLE = 1000
# FC, FP, items in flight per CU, cycles per K step (alone, per item sharing the CU), K split
PW_SHAPES = ((2, 2, 8, 470, 64, 1), (1, 1, 16, 300, 100, 1), (2, 2, 1, 470, 256, 4))
# block forms: (32-channel blocks, 32-pixel blocks) of a workgroup's block, two blocks per CU
PWB_SHAPES = ((4, 4), (2, 8))
C_PWB_BLOCK = 4000
PWB_BYTES_PER_CYCLE = 25
C_PW_SK = 2000
C_PW_ITEM = 2500
C_PW_RES = 1000
PW_HBM_BYTES_PER_CYCLE = 2000
# block 3x3 kernel: (64-channel waves along the channels, input channels per activation block,
# 32-pixel blocks of a wave's part)
C3_SHAPES = ((2, 32, 2), (2, 64, 2), (1, 32, 2), (1, 64, 2), (2, 32, 4))
C3_WAVES = 8
C3_LOAD_WAVES = 4
C3_MAX_ACT_LOADS = 16
C3_EPI_BYTES = C3_WAVES * 64 * 72 * 2
C_C3_ITEM = 10000
C_C3_SHORT_K = 6000
C3_MMA_TENTHS = 16
C3_BYTES_PER_CYCLE = 25
C3_SHALLOW_RING = 300

WG_THREADS = 512
WAVES = 8
MMA_WAVES = 4
LOAD_THREADS = 256
STAGE_VECS = 8
CPAD = 8
MAX_STAGES = 8
LDS_PER_CU = 160 * 1024

VAR_FC = (2, 1, 1, 1)
VAR_FP = (2, 4, 2, 2)
VAR_OCC = (1, 1, 1, 2)
TILE_H = (2, 4, 7, 8, 14, 16)
TILE_W = (4, 7, 8, 14, 16, 28, 32)

CONV, POOL, DW = 0, 1, 2


def cdiv(a, b):
    return -(-a // b)


def rup(a, b):
    return cdiv(a, b) * b


class NetInfo:
    """Shapes and packing parameters of every layer (plain shape inference)."""

    def __init__(self, net):
        self.layers = net["layers"]
        self.cache = {}
        n = len(self.layers)
        self.src, self.ish, self.osh = [0] * n, [None] * n, [None] * n
        self.cin_pad, self.ncb, self.nsteps, self.im2col = [0] * n, [0] * n, [0] * n, [False] * n
        self.rowfold = [False] * n
        for i, L in enumerate(self.layers):
            s = L["input_from"] if L["input_from"] >= 0 else i - 1
            self.src[i] = s
            h, w, c = (net["in_h"], net["in_w"], net["in_c"]) if s < 0 else self.osh[s]
            self.ish[i] = (h, w, c)
            op = L["op"]
            if op in ("conv", "dwconv", "maxpool"):
                ho = (h + 2 * L["pad"] - L["kh"]) // L["stride"] + 1
                wo = (w + 2 * L["pad"] - L["kw"]) // L["stride"] + 1
                self.osh[i] = (ho, wo, L["cout"])
            else:
                self.osh[i] = (1, 1, L["cout"])
            if op in ("conv", "fc"):
                narrow = op == "conv" and L["cin"] % 8 != 0
                self.rowfold[i] = narrow and L["cin"] <= 4 and L["stride"] % 2 == 0 and L["kw"] * 4 <= 128
                self.im2col[i] = narrow and not self.rowfold[i]
                k = L["kh"] * L["kw"] * L["cin"] if self.im2col[i] else L["cin"]
                if self.rowfold[i]:
                    k = L["kw"] * 4
                self.cin_pad[i] = rup(k, 32)
                self.ncb[i] = cdiv(L["cout"], 32)
                if self.rowfold[i]:
                    self.nsteps[i] = (self.cin_pad[i] // 16) * L["kh"]
                elif self.im2col[i]:
                    self.nsteps[i] = self.cin_pad[i] // 16
                else:
                    self.nsteps[i] = (self.cin_pad[i] // 32) * L["kh"] * L["kw"] * 2
            elif op == "dwconv":
                self.cin_pad[i] = rup(L["cin"], 8)

    def escapes(self, j):
        """Is tensor j read by a layer other than j+1, or added as a residual by any layer?"""
        for k, L in enumerate(self.layers):
            if L["residual_from"] == j:
                return True
            if k != j + 1 and self.src[k] == j:
                return True
        return False


def group_stages(ni, first, last):
    """Stage list [(layer, kind, pool2, pool_layer)] of a legal group, 'fc' / 'gap' for the
    single-layer special kernels, or None if layers [first, last] cannot form a group."""
    Ls = ni.layers
    if Ls[first]["op"] in ("fc", "gavgpool"):
        if first != last:
            return None
        return "fc" if Ls[first]["op"] == "fc" else "gap"
    st = []
    i = first
    while i <= last:
        L = Ls[i]
        op = L["op"]
        if op in ("fc", "gavgpool"):
            return None
        if i > first and ni.src[i] != i - 1:
            return None
        rf = L["residual_from"]
        if first <= rf <= last:
            return None
        if rf >= 0 and (op != "conv" or i != last):
            return None
        if i < last and ni.escapes(i):
            return None
        pool2, pool_layer = 0, -1
        if op == "conv":
            kind = CONV
            if L["cout"] % 4:
                return None
            if i + 1 <= last:
                P = Ls[i + 1]
                if (P["op"] == "maxpool" and P["kh"] == 2 and P["kw"] == 2 and P["stride"] == 2
                        and P["pad"] == 0 and ni.src[i + 1] == i and ni.osh[i][0] % 2 == 0
                        and ni.osh[i][1] % 2 == 0 and rf < 0):
                    if i + 1 < last and ni.escapes(i + 1):
                        return None
                    pool2, pool_layer = 1, i + 1
        elif op == "dwconv":
            kind = DW
            if L["cin"] % 8:
                return None
        else:
            kind = POOL
            if L["cin"] % 8 or L["pad"] >= L["kh"]:
                return None
        st.append((i, kind, pool2, pool_layer))
        i += 2 if pool2 else 1
    if len(st) > MAX_STAGES:
        return None
    for k in range(1, len(st)):
        if st[k][1] == CONV and st[k - 1][1] != CONV and Ls[st[k][0]]["cin"] % 32:
            return None
    return st


def build_group(ni, specs, batch, th, tw, variant, nslices, slice_c, stream0, kc, ksplit, max_lds):
    """Per-tile quantities of one candidate tiling, or None if it does not fit.
    Returns (ntiles, lds_bytes, tile_cycles, tile_hbm_bytes, tile_l2_bytes, tile_mma_cycles)."""
    Ls = ni.layers
    ns = len(specs)
    FC, FP = VAR_FC[variant], VAR_FP[variant]
    lfirst = specs[0][0]
    llast = specs[-1][3] if specs[-1][2] else specs[-1][0]
    in_h, in_w, in_c = ni.ish[lfirst]
    out_h, out_w, out_c = ni.osh[llast]
    ntiles = batch * cdiv(out_h, th) * cdiv(out_w, tw) * nslices
    S = [dict() for _ in range(ns)]
    my, oy, mx, ox, h, w = 1, 0, 1, 0, th, tw
    for s in range(ns - 1, -1, -1):
        li, kind, pool2, _ = specs[s]
        L = Ls[li]
        st = S[s]
        st["kind"], st["pool2"] = kind, pool2
        if pool2:
            my, oy, mx, ox, h, w = my * 2, oy * 2, mx * 2, ox * 2, h * 2, w * 2
        st["cin"], st["cout"] = L["cin"], L["cout"]
        kh, kw, stride, pad = L["kh"], L["kw"], L["stride"], L["pad"]
        st["rh"], st["rw"], st["oy_off"], st["ox_off"] = h, w, oy, ox
        st["ih"], st["iw"] = (h - 1) * stride + kh, (w - 1) * stride + kw
        my, oy = my * stride, oy * stride - pad
        mx, ox = mx * stride, ox * stride - pad
        h, w = st["ih"], st["iw"]
        st["im2col"] = 0
        st["kh"], st["kw"] = kh, kw
        if kind == CONV and ni.rowfold[li]:
            if s != 0 or stream0:
                return None
            st.update(im2col=2, im_kh=kh, im_kw=kw, im_stride=stride, im_cin=L["cin"], kw=1,
                      iw=rup(st["iw"], 2))
        elif kind == CONV and ni.im2col[li]:
            if s != 0 or stream0:
                return None
            st.update(im2col=1, im_kh=kh, im_kw=kw, im_stride=stride, im_cin=L["cin"], kh=1, kw=1,
                      ih=st["rh"], iw=st["rw"])
        if kind == CONV:
            st["kc"] = kc if (s == 0 and stream0) else 32
            st["cin_pad"], st["ncb"], st["nsteps"] = ni.cin_pad[li], ni.ncb[li], ni.nsteps[li]
            if st["kc"] not in (32, 64, 128):
                return None
            if st["cin_pad"] % st["kc"]:
                return None
            if st["kc"] != 32 and L["cin"] % 8:
                return None
        else:
            st["kc"], st["cin_pad"], st["ncb"], st["nsteps"] = 8, rup(L["cin"], 8), 0, 0
    if nslices > 1:
        if any(S[s]["kind"] == CONV for s in range(1, ns)):
            return None
        if S[0]["kind"] == CONV and slice_c % 32:
            return None
        if slice_c % 8:
            return None
        cslice = S[0]["cout"] if S[0]["kind"] == CONV else S[0]["cin"]
        if nslices * slice_c < cslice:
            return None
    if batch * in_h * in_w * in_c >= 1 << 31:
        return None
    if batch * (out_h + 32) * (out_w + 32) * out_c >= 1 << 31:
        return None
    chan_local = slice_c if nslices > 1 else 0
    area = [0, 0]
    for s in range(ns):
        st = S[s]
        if st["kind"] == CONV and st["im2col"] == 2:
            cs = 4
        elif st["kind"] == CONV:
            cs = st["kc"] + CPAD if (s == 0 and stream0) else st["cin_pad"] + CPAD
        else:
            cs = rup(chan_local if chan_local else st["cin"], 8) + CPAD
        sz = st["ih"] * st["iw"] * cs
        if st["kind"] == CONV and st["im2col"] == 2:
            sz += 32
        if s == 0 and stream0:
            sz *= 2
            if st["ih"] * st["iw"] * (st["kc"] // 8) > STAGE_VECS * LOAD_THREADS:
                return None
        area[s & 1] = max(area[s & 1], sz)
    sl = S[ns - 1]
    if sl["kind"] == CONV:
        c = chan_local if chan_local else sl["cout"]
        ph = sl["rh"] // 2 if sl["pool2"] else sl["rh"]
        pw = sl["rw"] // 2 if sl["pool2"] else sl["rw"]
        # the output tile overwrites the last stage's input where no wave has a second work item
        n_pg = cdiv(cdiv(sl["rh"] * sl["rw"], 32), FP)
        cbs = min(sl["ncb"], slice_c // 32) if nslices > 1 else sl["ncb"]
        alias = (ns == 1 and stream0) or n_pg * cdiv(cbs, FC) <= WAVES
        a = (ns - 1 if alias else ns) & 1
        area[a] = max(area[a], ph * pw * (rup(c, 8) + CPAD))
    for s in range(ns - 1):
        p, c = S[s], S[s + 1]
        ph = p["rh"] // 2 if p["pool2"] else p["rh"]
        pw = p["rw"] // 2 if p["pool2"] else p["rw"]
        if ph != c["ih"] or pw != c["iw"]:
            return None
        if p["pool2"] and ((p["oy_off"] & 1) or (p["ox_off"] & 1) or (p["rh"] & 1) or (p["rw"] & 1)):
            return None
    if sl["pool2"] and th * 2 != sl["rh"]:
        return None
    lds_halfs = area[0] + area[1]
    if ksplit > 1:
        # K of a single resident CONV stage split over `ksplit` waves per work item: register tile
        # of at most 32 x 64, chunks divisible, one pass of work items, partial sums of all 8 waves
        # in LDS (fp32)
        st = S[0]
        if ksplit not in (2, 4, 8) or ns != 1 or st["kind"] != CONV or stream0 or st["im2col"] or FC * FP > 2:
            return None
        if (st["cin_pad"] // 32) % ksplit:
            return None
        n_pg = cdiv(cdiv(st["rh"] * st["rw"], 32), FP)
        cbs = min(st["ncb"], slice_c // 32) if nslices > 1 else st["ncb"]
        if n_pg * cdiv(cbs, FC) * ksplit > WAVES:
            return None
        lds_halfs = rup(lds_halfs, 8) + WAVES * FC * FP * 16 * 64 * 2
    lds_bytes = lds_halfs * 2
    if lds_bytes > max_lds:
        return None

    # ---- cycles one workgroup spends on one tile ----
    cyc, l2, mma_total = C_TILE, 0, 0
    s0 = S[0]
    cin0 = chan_local if (s0["kind"] != CONV and chan_local) else s0["cin"]
    if stream0:
        cyc += C_LAT
    elif s0["kind"] == CONV and s0["im2col"] == 2:
        cyc += C_LAT + cdiv(s0["ih"] * s0["iw"], WG_THREADS) * C_ROWFOLD
    elif s0["kind"] == CONV and s0["im2col"]:
        cyc += C_LAT + cdiv(s0["rh"] * s0["rw"] * s0["im_kh"], WG_THREADS) * s0["im_kw"] * s0["im_cin"] * C_IM2COL
    else:
        cfill = s0["cin_pad"] if s0["kind"] == CONV else rup(cin0, 8)
        cyc += C_LAT + cdiv(s0["ih"] * s0["iw"] * (cfill // 8), WG_THREADS) * C_STAGE_VEC
    for s in range(ns):
        st = S[s]
        npix = st["rh"] * st["rw"]
        if st["kind"] == CONV:
            n_pg = cdiv(cdiv(npix, 32), FP)
            cbs = min(st["ncb"], slice_c // 32) if nslices > 1 else st["ncb"]
            nitems = n_pg * cdiv(cbs, FC) * ksplit          # K slices run like work items
            streaming = s == 0 and stream0
            mma_waves = MMA_WAVES if streaming else WAVES
            if streaming and nitems > mma_waves:
                return None
            mma = cdiv(nitems, 4) * (st["nsteps"] // ksplit) * FC * FP * MFMA_CYCLES * (13 if FP >= 4 else 20) // 10
            if streaming:
                nrounds = st["cin_pad"] // st["kc"]
                vecs = cdiv(st["ih"] * st["iw"] * (st["kc"] // 8), LOAD_THREADS)
                mma = max(mma, nrounds * (C_ROUND + vecs * C_ROUND_VEC)) + nrounds * C_BARRIER
            mma_total += mma
            cyc += mma + cdiv(nitems, mma_waves) * FC * FP * C_EPI + (C_KSPLIT if ksplit > 1 else 0)
            l2 += nitems * FC * (st["nsteps"] // ksplit) * 1024
        else:
            c = chan_local if chan_local else st["cout"]
            items = npix * cdiv(c, 8)
            cyc += cdiv(items, WG_THREADS) * (st["kh"] * st["kw"]) * C_VALU + C_STAGE
    cout_l = min(chan_local, out_c) if chan_local else out_c
    has_res = 1 if Ls[specs[-1][0]]["residual_from"] >= 0 else 0
    if sl["kind"] == CONV:
        cyc += cdiv(th * tw * cdiv(cout_l, 8), WG_THREADS) * C_STORE_VEC + C_STORE + has_res * C_LAT
    hbm = s0["ih"] * s0["iw"] * cin0 * 2 + th * tw * cout_l * 2 * (1 + has_res)
    if s0["kind"] == CONV and s0["im2col"] == 2:
        hbm = s0["ih"] * s0["iw"] * s0["im_cin"] * 2 + th * tw * cout_l * 2
    elif s0["kind"] == CONV and s0["im2col"]:
        hbm = s0["rh"] * s0["rw"] * s0["im_stride"] * s0["im_stride"] * s0["im_cin"] * 2 + th * tw * cout_l * 2
    return ntiles, lds_bytes, cyc, hbm, l2, mma_total


def tiling_cost_ps(built, budget, variant):
    ntiles, lds_bytes, cyc, hbm, l2, mma_total = built
    occ = max(1, min(VAR_OCC[variant], LDS_PER_CU // max(lds_bytes, 1)))
    cu = min(budget, ntiles)
    wg = min(ntiles, budget * occ)
    conc = cdiv(wg, cu)
    tiles_cu = cdiv(ntiles, cu)
    # latency chains outside the MFMA loops: paid in full by a workgroup alone on its CU, filled in
    # by a second workgroup down to the time the shared matrix pipes are busy
    tile = mma_total + (cyc - mma_total) * 5 // 4
    compute = tiles_cu * (max(mma_total, tile * 3 // 5) if conc >= 2 else tile)
    bw = min(CU_BYTES_PER_CYCLE, max(1, HBM_BYTES_PER_CYCLE // cu))
    mem = tiles_cu * (hbm // bw + l2 // L2_BYTES_PER_CYCLE)
    return (C_LAUNCH + max(compute, mem)) * PS_PER_CYCLE


def candidates(ni, specs):
    """Every tiling the tuner considers for a group: (th, tw, variant, nslices, slice_c,
    stream0, kc, ksplit)."""
    Ls = ni.layers
    llast = specs[-1][3] if specs[-1][2] else specs[-1][0]
    out_h, out_w, _ = ni.osh[llast]
    l0 = specs[0][0]
    conv0 = specs[0][1] == CONV
    later_conv = any(sp[1] == CONV for sp in specs[1:])
    any_conv = conv0 or later_conv
    for th in TILE_H:
        if th > out_h and th != TILE_H[0] and th - out_h >= 4:
            continue
        for tw in TILE_W:
            if tw > out_w and tw != TILE_W[0] and tw - out_w >= 4:
                continue
            if th * tw > 512:
                continue
            for variant in range(4):
                if not any_conv and variant not in (0, 3):
                    continue
                if conv0:
                    ncb, fc = ni.ncb[l0], VAR_FC[variant]
                    wide = Ls[l0]["cin"] % 8 == 0
                    for stream0 in (1, 0):
                        kc = 32
                        while kc <= (128 if (stream0 and wide) else 32):
                            if ni.cin_pad[l0] % kc == 0:
                                yield th, tw, variant, 1, 0, stream0, kc, 1
                                if not stream0 and len(specs) == 1 and fc * VAR_FP[variant] <= 2:
                                    for ks in (2, 4, 8):
                                        yield th, tw, variant, 1, 0, 0, 32, ks
                                        for cg in (1, 2, 4):
                                            sc = fc * cg * 32
                                            if sc < ncb * 32:
                                                yield th, tw, variant, cdiv(ncb * 32, sc), sc, 0, 32, ks
                                if not later_conv and stream0:
                                    for cg in (1, 2, 4):
                                        sc = fc * cg * 32
                                        if sc < ncb * 32:
                                            yield th, tw, variant, cdiv(ncb * 32, sc), sc, 1, kc, 1
                            kc *= 2
                else:
                    yield th, tw, variant, 1, 0, 0, 32, 1
                    if not later_conv:
                        sc = 32
                        while sc < Ls[l0]["cin"]:
                            yield th, tw, variant, cdiv(Ls[l0]["cin"], sc), sc, 0, 32, 1
                            sc *= 2


def pw_cost(ni, i, batch, budget):
    """Cost of a single 1x1 convolution on the barrier-free pointwise kernel, or None if it does
    not apply (needs 1x1, no padding, cin % 32 == 0, cout % 8 == 0)."""
    L = ni.layers[i]
    if L["op"] != "conv" or L["kh"] != 1 or L["kw"] != 1 or L["pad"] != 0:
        return None
    if L["cin"] % 32 or L["cout"] % 8:
        return None
    ih, iw, ic = ni.ish[i]
    oh, ow, oc = ni.osh[i]
    if batch * ih * iw * ic >= 1 << 31 or batch * oh * ow * oc >= 1 << 31:
        return None
    m = batch * oh * ow
    has_res = 1 if L["residual_from"] >= 0 else 0
    nsteps = ni.nsteps[i]
    nbytes = m * L["cin"] * 2 + m * L["cout"] * 2 * (1 + has_res) + ni.ncb[i] * nsteps * 1024
    mem = nbytes // min(PW_HBM_BYTES_PER_CYCLE, budget * CU_BYTES_PER_CYCLE)
    best = None
    for fc, fp, w, step0, step_wave, ks in PW_SHAPES:
        if ks > 1 and (nsteps % ks or nsteps < 16):
            continue
        items = cdiv(m, 32 * fp) * cdiv(ni.ncb[i], fc)
        items_cu = cdiv(items, budget)
        step = max(step0, min(items_cu, w) * step_wave)
        item = C_PW_ITEM + (nsteps // ks) * step + (C_PW_SK if ks > 1 else 0) + has_res * C_PW_RES
        stream = items_cu * nsteps * (fc + fp) * 1024 // PWB_BYTES_PER_CYCLE
        compute = max(cdiv(items_cu, w) * item, stream)
        c = (C_LAUNCH + max(compute, mem)) * PS_PER_CYCLE
        if best is None or c < best:
            best = c
    for k, (bc, bp) in enumerate(PWB_SHAPES):
        # 128 x 128 blocks for more than 64 output channels, 64 x 256 otherwise
        if (k == 0) != (ni.ncb[i] >= 3):
            continue
        items = cdiv(m, 32 * bp) * cdiv(ni.ncb[i], bc)
        items_cu = cdiv(items, budget)
        rounds = cdiv(items_cu, 2)
        frag_bytes = items_cu * nsteps * (bc + bp) * 1024
        compute = rounds * (C_PWB_BLOCK + has_res * C_PW_RES) + frag_bytes // PWB_BYTES_PER_CYCLE
        c = (C_LAUNCH + max(compute, mem)) * PS_PER_CYCLE
        if best is None or c < best:
            best = c
    return best


def c3_cost(ni, specs, batch, budget, max_lds):
    """Cost of a single 3x3 stride-1 pad-1 convolution (with its folded 2x2 pool, if any) on the
    block 3x3 kernel: cheapest of its shapes and pixel tiles, or None where it does not apply."""
    if len(specs) != 1 or specs[0][1] != CONV:
        return None
    i, pool2 = specs[0][0], specs[0][2]
    L = ni.layers[i]
    if L["op"] != "conv" or L["kh"] != 3 or L["kw"] != 3 or L["stride"] != 1 or L["pad"] != 1:
        return None
    if L["cin"] % 32 or L["cout"] % 8:
        return None
    ih, iw, ic = ni.ish[i]
    oh, ow, oc = ni.osh[i]
    if batch * ih * iw * ic >= 1 << 31 or batch * oh * ow * oc >= 1 << 31:
        return None
    has_res = 1 if L["residual_from"] >= 0 else 0
    m = batch * oh * ow
    nbytes = m * L["cin"] * 2 + (m // 4 if pool2 else m) * L["cout"] * 2 * (1 + has_res) \
        + ni.ncb[i] * ni.nsteps[i] * 1024
    mem = nbytes // min(PW_HBM_BYTES_PER_CYCLE, budget * CU_BYTES_PER_CYCLE)
    kt = L["cin"] // 16
    best = None
    for wc, ach, fp in C3_SHAPES:
        if L["cin"] % ach:
            continue
        for th in TILE_H:
            if th > oh and th != TILE_H[0] and th - oh >= 4:
                continue
            for tw in TILE_W:
                if tw > ow and tw != TILE_W[0] and tw - ow >= 4:
                    continue
                if th * tw > 32 * fp * (C3_WAVES // wc) or (pool2 and ((th | tw) & 1)):
                    continue
                npxh = (th + 2) * (tw + 2)
                na_i = cdiv(npxh, 512 // ach)
                if cdiv(na_i, C3_LOAD_WAVES) > C3_MAX_ACT_LOADS:
                    continue
                act, wstage = 2 * na_i * 1024, 9 * 2 * wc * 1024
                nst = min(4, (max_lds - 1024 - act) // wstage)
                if nst < 2 or max(act + nst * wstage + 1024, C3_EPI_BYTES) > max_lds:
                    continue
                items = batch * cdiv(oh, th) * cdiv(ow, tw) * cdiv(ni.ncb[i], 2 * wc)
                items_cu = cdiv(items, budget)
                stage = max(9 * 2 * fp * MFMA_CYCLES * 2 * C3_MMA_TENTHS // 10,
                            (wstage + npxh * 32) // C3_BYTES_PER_CYCLE)
                if nst == 2:
                    stage += C3_SHALLOW_RING
                compute = items_cu * (C_C3_ITEM + (C_C3_SHORT_K if kt < 8 else 0) + has_res * C_PW_RES + kt * stage)
                c = (C_LAUNCH + max(compute, mem)) * PS_PER_CYCLE
                if best is None or c < best:
                    best = c
    return best


def group_cost(net, batch, first, last, budget, max_lds=LDS_PER_CU, ni=None):
    """Cost in picoseconds of running layers [first, last] as one group on `budget` CUs, or None."""
    ni = ni or NetInfo(net)
    specs = group_stages(ni, first, last)
    if specs is None:
        return None
    if specs == "fc":
        nbb = cdiv(batch, 32)
        ncb, nsteps = ni.ncb[first], ni.nsteps[first]
        best = (C_LAUNCH + C_LAT + ncb * nsteps * 1024 * nbb // FC_BYTES_PER_CYCLE) * PS_PER_CYCLE
        # split-K form: pairs of channel blocks, K in 2 / 4 / 8 slices, a second launch adds them
        for ks in (2, 4, 8):
            if cdiv(ncb, 2) * ks > 256 or nsteps < 64 * ks:
                continue
            intake = 3 * cdiv(nsteps, ks) * 1024 * nbb // PWB_BYTES_PER_CYCLE
            hbm = ncb * nsteps * 1024 * nbb // FC_SPLIT_HBM_BYTES_PER_CYCLE
            best = min(best, (2 * C_LAUNCH + C_LAT + max(intake, hbm)) * PS_PER_CYCLE)
        return best
    if specs == "gap":
        h, w, c = ni.ish[first]
        return (C_LAUNCH + C_LAT + batch * h * w * c * 2 // GAP_BYTES_PER_CYCLE) * PS_PER_CYCLE
    key = (first, last, batch, max_lds)
    built = ni.cache.get(key)
    if built is None:
        built = []
        for cand in candidates(ni, specs):
            b = build_group(ni, specs, batch, *cand, max_lds)
            if b is not None:
                built.append((b, cand[2]))
        ni.cache[key] = built
    best = None
    for b, variant in built:
        c = tiling_cost_ps(b, budget, variant)
        if best is None or c < best:
            best = c
    if first == last:
        pc = pw_cost(ni, first, batch, budget)
        if pc is not None and (best is None or pc < best):
            best = pc
    cc = c3_cost(ni, specs, batch, budget, max_lds)
    if cc is not None and (best is None or cc < best):
        best = cc
    return best


def cost_table(net, batch, budgets, max_lds=LDS_PER_CU):
    """cost[(first, last, budget)] for every contiguous range (None = cannot be a group)."""
    ni = NetInfo(net)
    n = len(net["layers"])
    return {(f, l, b): group_cost(net, batch, f, l, b, max_lds, ni)
            for f in range(n) for l in range(f, n) for b in budgets}
