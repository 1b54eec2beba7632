"""The full-network configuration: ResNet-18 at 224x224 with the first conv and the
classifier in fp32 and every other conv RTN-ternary (weights and activations), BN folded
into the conv epilogues (appendix "Layer Order"; Table 4 lists the ternary layers).

Only orchestration lives here.  The stem (7x7/2 conv, BN, ReLU, 3x3/2 max-pool) and the
head (average pool, FC) are plain torch fp32 ops -- the paper keeps them in full precision
and they are outside the ternary library.  The trunk, the 8 residual blocks of 19 ternary
convs, runs through the C ABI: one rtn_ternarize_pack of the trunk input, then per block
conv1 with the ternarizing epilogue, the 1x1/stride-2 shortcut conv where the block
changes shape, and conv2 with the block-tail epilogue (shortcut add, ReLU, fp32 block
output and the next block's codes).  A block computes
    out = relu(bn2(tconv2(T(bn1(relu(tconv1(T(x))))))) + shortcut(x)),
T = ternarize at the network's activation threshold; the paper's figure of the block is
not in its text, so this topology is this repository's reading of it."""
import numpy as np
import torch

from . import binding as B
from . import workloads as wl


class TernaryResNet18:
    def __init__(self, params, batch, device="cuda:0", fmt=B.RTN_CODE_FP4):
        self.batch, self.dev, self.fmt = batch, device, fmt
        self.blocks = wl.resnet18_block_topology()
        self.delta = float(params["delta_a"])
        d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
        g = lambda v: (float(v) if np.ndim(v) == 0 else d(np.asarray(v, np.float32)))
        self.stem_w, self.fc_w, self.fc_b = d(params["stem_w"]), d(params["fc_w"]), d(params["fc_b"])
        self.stem_scale = d(params["stem_scale"]).view(1, -1, 1, 1)
        self.stem_shift = d(params["stem_shift"]).view(1, -1, 1, 1)
        tail = {i2 for _, i2, _ in self.blocks}
        self.L = []
        for i, p in enumerate(params["layers"]):     # S0, offline: weight codes, tap sums, constant tables
            sh = p["sh"]
            dw = np.asarray(p["dw"])
            cw, pw = B.ternarize_pack(d(p["w"]), g(-dw), g(dw), fmt)
            # conv1 of a block: conv -> ReLU -> BN; conv2 and the shortcut conv: conv -> BN
            ep = B.Epilogue(g(p["aa"]), g(p["ba"]), g(p["aw"]), g(p["bw"]), None, pw,
                            relu=(i not in tail and sh.k == 3), bn_scale=d(p["bs"]), bn_shift=d(p["bh"]))
            ws = torch.empty(B.conv2d_workspace_bytes(sh.O, sh.k, sh.k, sh.pad), dtype=torch.uint8, device=device)
            B.conv2d_prepare_constants(sh.C, sh.O, sh.k, sh.k, sh.pad, ep, ws)
            self.L.append(dict(sh=sh, cw=cw, pw=pw, ep=ep, ws=ws,
                               codes_in=self._codes(batch, sh.H, sh.C),
                               y=torch.empty((batch, sh.O, sh.OH, sh.OH), dtype=torch.float32, device=device)
                               if (i in tail or sh.k == 1) else None))
        self.last_codes = self._codes(batch, 7, 512)

    def _codes(self, n, hw, channels):
        """An empty code tensor [n, hw, hw, row] in this network's code format."""
        kp = B.padded_k(channels, self.fmt)
        if self.fmt == B.RTN_CODE_I8:
            return torch.empty((n, hw, hw, kp), dtype=torch.int8, device=self.dev)
        return torch.empty((n, hw, hw, kp // 2), dtype=torch.uint8, device=self.dev)

    def stem(self, images):
        x = torch.nn.functional.conv2d(images, self.stem_w, stride=2, padding=3)
        x = torch.relu(x * self.stem_scale + self.stem_shift)
        return torch.nn.functional.max_pool2d(x, 3, stride=2, padding=1).contiguous()

    def head(self, x):
        return torch.nn.functional.linear(x.mean(dim=(2, 3)), self.fc_w, self.fc_b)

    def trunk(self, x0, keep=None):
        """x0: fp32 [batch,64,56,56] -> fp32 [batch,512,7,7].  keep: optional list that receives
        per block (codes into conv1, codes into conv2, fp32 block output)."""
        Nb, lo, hi = self.batch, -self.delta, self.delta
        B.ternarize_pack(x0, lo, hi, self.fmt, codes=self.L[0]["codes_in"], want_sum=False)
        cur_x, cur_codes = x0, self.L[0]["codes_in"]
        for bi, (i1, i2, ids) in enumerate(self.blocks):
            l1, l2 = self.L[i1], self.L[i2]
            s1, s2 = l1["sh"], l2["sh"]
            B.ternary_conv2d_ternarize(cur_codes, l1["cw"], Nb, s1.C, s1.H, s1.H, s1.O, s1.k, s1.k, s1.stride,
                                       s1.pad, l1["ep"], lo, hi, codes_out=l2["codes_in"], workspace=l1["ws"],
                                       fmt=self.fmt)
            if ids is None:
                res = cur_x
            else:
                ld = self.L[ids]
                sd = ld["sh"]
                B.ternary_conv2d(cur_codes, ld["cw"], Nb, sd.C, sd.H, sd.H, sd.O, sd.k, sd.k, sd.stride, sd.pad,
                                 B.RTN_PAD_TRUE_ZERO, ep=ld["ep"], y_out=ld["y"], workspace=ld["ws"], fmt=self.fmt)
                res = ld["y"]
            nxt = self.L[self.blocks[bi + 1][0]]["codes_in"] if bi + 1 < len(self.blocks) else self.last_codes
            B.ternary_conv2d_ternarize(l2["codes_in"], l2["cw"], Nb, s2.C, s2.H, s2.H, s2.O, s2.k, s2.k, s2.stride,
                                       s2.pad, l2["ep"], lo, hi, codes_out=nxt, workspace=l2["ws"], residual=res,
                                       relu_out=True, y_out=l2["y"], fmt=self.fmt)
            if keep is not None:
                keep.append((cur_codes, l2["codes_in"], l2["y"]))
            cur_x, cur_codes = l2["y"], nxt
        return cur_x

    def forward(self, images):
        return self.head(self.trunk(self.stem(images)))

    def trunk_macs(self):
        return sum(l["sh"].macs(self.batch) for l in self.L)

    def trunk_bytes(self):
        """Algorithmic HBM bytes of one trunk pass: what each launch must read and write
        once (fp32 trunk input, int8 codes, filters, fp32 shortcut tensors, fp32 block outputs)."""
        Nb = self.batch
        cb = (lambda ch: B.padded_k(ch, self.fmt) // (2 if self.fmt == B.RTN_CODE_FP4 else 1))   # bytes of a code row
        total = Nb * 56 * 56 * (64 * 4 + cb(64))                 # the one pack: fp32 in, codes out
        for i1, i2, ids in self.blocks:
            for i, kind in ((i1, "c1"), (ids, "ds"), (i2, "c2")):
                if i is None:
                    continue
                sh = self.L[i]["sh"]
                cin = Nb * sh.H * sh.H * cb(sh.C) + sh.O * sh.k * sh.k * cb(sh.C)
                outs = Nb * sh.O * sh.OH * sh.OH
                codes_out = Nb * sh.OH * sh.OH * cb(sh.O)
                if kind == "c1":
                    total += cin + codes_out
                elif kind == "ds":
                    total += cin + outs * 4                    # fp32 shortcut out
                else:
                    total += cin + outs * (4 + 4) + codes_out  # residual in, fp32 block output + codes out
        return total
