"""A MinkUNet-style encoder-decoder assembled from the library's layers, written once
against a small backend interface so that the HIP library and the CPU oracle run the very
same graph.  Architecture (defined by this repository, not taken from any project):

  stem   conv3 8 -> 32, ReLU                                            (level 0)
  enc i  conv3 stride 2 c[i-1] -> c[i], ReLU; two residual blocks       (levels 1..4, c = 32, 64, 128, 256)
  dec i  transposed conv3 stride 2 -> d[i], ReLU; concat with the encoder output of that
         level; two residual blocks at d[i] (the first with a 1x1x1 projection on its skip
         path because the concat changed the width)                     (d = 128, 64, 32, 32)
  residual block: y = ReLU(conv3(ReLU(conv3(x))) + skip(x));  no normalisation layers.
"""
import numpy as np

ENC = [32, 32, 64, 128, 256]   # widths at levels 0..4
DEC = [128, 64, 32, 32]        # widths of decoder stages 1..4 (levels 3, 2, 1, 0)
C_FEAT = 8


def layer_shapes():
    """name -> (K, c_in, c_out) in execution order."""
    shapes = {"stem": (3, C_FEAT, ENC[0])}
    for i in range(1, 5):
        shapes[f"down{i}"] = (3, ENC[i - 1], ENC[i])
        for b in (1, 2):
            shapes[f"e{i}b{b}.c1"] = (3, ENC[i], ENC[i])
            shapes[f"e{i}b{b}.c2"] = (3, ENC[i], ENC[i])
    h = ENC[4]
    for i in range(1, 5):
        lvl = 4 - i
        d = DEC[i - 1]
        shapes[f"up{i}"] = (3, h, d)
        cat = d + ENC[lvl]
        shapes[f"d{i}b1.c1"] = (3, cat, d)
        shapes[f"d{i}b1.c2"] = (3, d, d)
        shapes[f"d{i}b1.proj"] = (1, cat, d)
        shapes[f"d{i}b2.c1"] = (3, d, d)
        shapes[f"d{i}b2.c2"] = (3, d, d)
        h = d
    return shapes


class Net:
    """Runs the graph on a backend `be` with
       conv(x, name, km) / dgrad(dy, name, km) / wgrad(x, dy, km) -> tensors,
       relu, add, add_relu, relu_bwd(dy, y), concat(a, b), split(d, ca) and
       kmaps be.sub[l], be.one[l], be.down[l], be.up[l]."""

    def __init__(self, be):
        self.be = be

    def _block(self, x, name, km3, km1, proj, tape):
        be = self.be
        h1 = be.relu(be.conv(x, name + ".c1", km3))
        h2 = be.conv(h1, name + ".c2", km3)
        skip = be.conv(x, name + ".proj", km1) if proj else x
        y = be.add_relu(h2, skip)
        tape.append(("block", name, km3, km1, proj, x, h1, y))
        return y

    def forward(self, x0):
        be, tape = self.be, []
        s_pre = be.conv(x0, "stem", be.sub[0])
        h = be.relu(s_pre)
        tape.append(("conv_relu", "stem", be.sub[0], x0, h))
        enc = [h]
        for i in range(1, 5):
            x = h
            h = be.relu(be.conv(x, f"down{i}", be.down[i - 1]))
            tape.append(("conv_relu", f"down{i}", be.down[i - 1], x, h))
            h = self._block(h, f"e{i}b1", be.sub[i], None, False, tape)
            h = self._block(h, f"e{i}b2", be.sub[i], None, False, tape)
            enc.append(h)
        for i in range(1, 5):
            lvl = 4 - i
            x = h
            u = be.relu(be.conv(x, f"up{i}", be.up[lvl]))
            tape.append(("conv_relu", f"up{i}", be.up[lvl], x, u))
            cat = be.concat(u, enc[lvl])
            tape.append(("concat", DEC[i - 1], lvl))
            h = self._block(cat, f"d{i}b1", be.sub[lvl], be.one[lvl], True, tape)
            h = self._block(h, f"d{i}b2", be.sub[lvl], None, False, tape)
        self.tape, self.n_enc = tape, len(enc)
        return h

    def backward(self, dy):
        """Returns (dW dict, dx0).  Gradients flowing into encoder outputs through the skip
        concatenations are accumulated per level."""
        be = self.be
        dW, d_enc = {}, {}
        g = dy
        # walk the tape backwards; remember which encoder level each stage output belongs to
        # (an encoder stage's output is the last block of that stage)
        enc_owner = {f"e{i}b2": i for i in range(1, 5)}
        for rec in reversed(self.tape):
            kind = rec[0]
            if kind == "block":
                _, name, km3, km1, proj, x, h1, y = rec
                if name in enc_owner and enc_owner[name] in d_enc:
                    g = be.add(g, d_enc.pop(enc_owner[name]))
                dz = be.relu_bwd(g, y)
                dW[name + ".c2"] = be.wgrad(h1, dz, km3)
                dh1 = be.relu_bwd(be.dgrad(dz, name + ".c2", km3), h1)
                dW[name + ".c1"] = be.wgrad(x, dh1, km3)
                dx = be.dgrad(dh1, name + ".c1", km3)
                if proj:
                    dW[name + ".proj"] = be.wgrad(x, dz, km1)
                    g = be.add(dx, be.dgrad(dz, name + ".proj", km1))
                else:
                    g = be.add(dx, dz)
            elif kind == "concat":
                _, ca, lvl = rec
                g, d_skip = be.split(g, ca)
                d_enc[lvl] = d_skip
            else:  # conv_relu
                _, name, km, x, y = rec
                if name == "stem" and 0 in d_enc:
                    g = be.add(g, d_enc.pop(0))
                dz = be.relu_bwd(g, y)
                dW[name] = be.wgrad(x, dz, km)
                g = be.dgrad(dz, name, km)
        return dW, g
