"""Turns a ``workloads.Model`` table plus host weights into what
``gpulet_run_model`` takes: device weights in the library's layouts and the
flat ``gpulet_layer`` array over numbered activation buffers.

Only marshalling happens here (layout permutations, buffer numbering, device
copies); no layer is computed.  torch provides device memory.

Layout conversions
  * activations (N, C, H, W) -> NHWC bf16,
  * convolution weights (K, C, R, S) -> KRSC bf16,
  * FC weights whose input is a (C, H, W) feature map: columns go from the
    channel-major flatten order to the NHWC one.

The model input is stored with its channel count padded with zeros, and the
first convolution's weights are padded to match; the extra channels contribute
exact zeros.  RGB stems (C = 3, a filter of 3, 5 or 7 rows, a multiple of 8
filters) are padded to 4 channels, the 8-byte pixels the library's stem kernel
stages; everything else (LeNet's C = 1 with 6 filters) to a multiple of 8, so
that it uses the same 16-byte gathers as every other layer.

Buffers are reused once their last reader has run, which keeps the working
set small enough to stay in the last-level cache between layers.  A concat
node costs nothing: its source convolutions store straight into channel
slices of the concatenated buffer.

Layers that can share a kernel launch are told so (``merge_siblings``, on by
default; see ``DeviceModel._stack_siblings``, ``_ride_pools`` and ``_chain_groups``): sibling convolutions
are stacked into one layer, an inception block's max pool rides along with
its 1x1 layers, and independent convolutions are chained into launch groups.
None of this changes what is computed, only how many launches it takes.
"""

import numpy as np
import torch

from . import gpulet


def to_device_bf16(a, device):
    """bfloat16-exact float32 numpy array -> torch bf16 tensor on ``device``."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device=device, dtype=torch.bfloat16)


def nchw_to_nhwc(x, device):
    return to_device_bf16(np.transpose(x, (0, 2, 3, 1)), device)


def nhwc_to_nchw(t):
    """Device NHWC tensor -> float64 numpy (N, C, H, W)."""
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64).transpose(0, 3, 1, 2)


def kcrs_to_krsc(w, device):
    return to_device_bf16(np.transpose(w, (0, 2, 3, 1)), device)


class DeviceModel:
    """A model resident on the GPU, ready for ``run`` / ``profile`` on a gpu-let.
    ``reuse=False`` gives every tensor its own buffer so intermediates can be
    read back after a run."""

    def __init__(self, model, params, device="cuda:0", reuse=True, fuse_pools=False, merge_siblings=True):
        self.model = model
        self.device = torch.device(device)
        self.in_shape = tuple(model.in_shape)
        self._keep = []  # device tensors the layer records point into
        nodes = [nd for nd in model.nodes]
        # channel padding of the model input (only convolutions may read it then)
        c_in = model.in_shape[0]
        readers = [nd for nd in nodes if nd.src == "x"]
        if not all(nd.op == "conv" for nd in readers):
            self.in_pad = 0
        elif c_in <= 4 and all(nd.attr["k"] in (3, 5, 7) and nd.attr["K"] % 8 == 0 for nd in readers):
            self.in_pad = 4 - c_in
        else:
            self.in_pad = (-c_in) % 8

        # channels of every named tensor, straight from the table
        chans = {"x": model.in_shape[0]}
        alias = {}  # concat source -> (concat tensor, channel offset, total channels)
        for nd in nodes:
            if nd.op == "conv":
                chans[nd.dst] = nd.attr["K"]
            elif nd.op in ("maxpool", "gavgpool", "dwconv"):
                chans[nd.dst] = chans[nd.src]
            elif nd.op == "fc":
                chans[nd.dst] = nd.attr["Out"]
            elif nd.op == "concat":
                total = sum(chans[s] for s in nd.src)
                off = 0
                for s in nd.src:
                    alias[s] = (nd.dst, off, total)
                    off += chans[s]
                chans[nd.dst] = total
        # A convolution whose K is not a multiple of 8 makes its reader gather 2-byte elements one by one
        # (the scalar-gather kernel: LeNet's 6 -> 16 layer took 13 us of the model's 41).  Where the
        # tensor goes nowhere but through at most one max pool into one plain convolution, the
        # producer gets zero filters up to the next multiple of 8 and the reader zero weights for
        # them: the extra channels are relu(0) = 0 and add exact zeros, every sum keeps its bits.
        self.k_pad = {}      # convolution name -> zero filters appended
        c_extra = {}         # tensor -> zero channels it carries
        all_readers = {}
        for nd in nodes:
            reads = list(nd.src) if nd.op == "concat" else [nd.src]
            if nd.op == "conv" and nd.attr["residual"]:
                reads.append(nd.attr["residual"])
            for t in reads:
                all_readers.setdefault(t, []).append(nd)
        for nd in nodes:
            if (nd.op != "conv" or nd.attr["K"] % 8 == 0 or nd.dst in alias or nd.dst == model.out or nd.attr["residual"]
                    or len(all_readers.get(nd.src, [])) != 1):
                continue
            chain, t = [], nd.dst
            rs = all_readers.get(t, [])
            if len(rs) == 1 and rs[0].op == "maxpool" and rs[0].dst != model.out:
                chain.append(rs[0])
                t = rs[0].dst
                rs = all_readers.get(t, [])
            if not (len(rs) == 1 and rs[0].op == "conv" and rs[0].src == t and not rs[0].attr["residual"]
                    and "in_slice" not in rs[0].attr):
                continue
            pad = (-nd.attr["K"]) % 8
            self.k_pad[nd.name] = pad
            c_extra[nd.dst] = pad
            chans[nd.dst] += pad
            for pool in chain:
                c_extra[pool.dst] = pad
                chans[pool.dst] += pad
        # With ``fuse_pools`` a 3x3 / stride 1 / pad 1 max pool whose only reader is a plain 1x1
        # convolution (the pooling branch of an inception block) runs inside that convolution's
        # kernel and the pooled tensor is never stored; ``fused_pools`` names the pool nodes that
        # disappeared this way.  Same bits either way.  Off by default: measured on the GoogLeNet
        # shape the fused kernel's chain of dependent depth slices costs more than the separate,
        # massively parallel pool kernel saves (batch 32: 0.565 against 0.560 ms, batch 1: 0.423
        # against 0.394 ms).
        self.fused_pools = []
        if fuse_pools:
            readers = {}
            for nd in nodes:
                reads = list(nd.src) if nd.op == "concat" else [nd.src]
                if nd.op == "conv" and nd.attr["residual"]:
                    reads.append(nd.attr["residual"])
                for t in reads:
                    readers.setdefault(t, []).append(nd)
            moved, kept = {}, []
            for nd in nodes:
                a = nd.attr
                if (nd.op == "maxpool" and (a["k"], a["stride"], a["pad"]) == (3, 1, 1) and nd.dst != model.out
                        and nd.src != "x" and chans[nd.src] % 8 == 0):
                    rs = readers.get(nd.dst, [])
                    if (len(rs) == 1 and rs[0].op == "conv" and rs[0].src == nd.dst and not rs[0].attr["residual"]
                            and (rs[0].attr["k"], rs[0].attr["stride"], rs[0].attr["pad"]) == (1, 1, 0)):
                        moved[nd.dst] = nd.src
                        self.fused_pools.append(nd.name)
                        continue
                if nd.op == "conv" and nd.src in moved:
                    nd = nd._replace(src=moved[nd.src], attr=dict(a, pre_pool=3))
                kept.append(nd)
            nodes = kept
        # Fewer launches: stacked sibling layers, pools riding along, launch groups (the passes below).
        self.merged, self.side_pools, self.groups = [], [], []
        if merge_siblings:
            nodes = self._stack_siblings(nodes, chans, alias, model)
            nodes = self._ride_pools(nodes, chans, alias, model)
            nodes = self._chain_groups(nodes, alias)
        producers = {nd.dst: nd for nd in nodes}
        for s in alias:
            if producers[s].op != "conv":
                raise ValueError("concat source %r must be produced by a convolution" % s)

        def storage(t):  # the tensor whose buffer holds t
            return alias[t][0] if t in alias else t

        # last node index at which each storage tensor is read
        last_use = {}
        for i, nd in enumerate(nodes):
            reads = list(nd.src) if nd.op == "concat" else [nd.src]
            if nd.op == "conv" and nd.attr["residual"]:
                reads.append(nd.attr["residual"])
            for t in reads:
                last_use[storage(t)] = i
            # A 2x2 / stride 2 max pool right behind a convolution may be computed by that convolution's
            # launch (the library decides per launch), which then writes the pool's buffer while it
            # still reads its own input: that input stays allocated until the pool is done.
            if (nd.op == "maxpool" and (nd.attr["k"], nd.attr["stride"], nd.attr["pad"]) == (2, 2, 0) and i > 0
                    and nodes[i - 1].op == "conv" and nodes[i - 1].dst == nd.src):
                last_use[storage(nodes[i - 1].src)] = max(last_use.get(storage(nodes[i - 1].src), 0), i)
        last_use[storage(model.out)] = len(nodes)

        buf_of = {"x": 0, storage(model.out): 1}
        free, n_bufs = [], 2
        layers = []
        self.tensor_buf = {}
        for i, nd in enumerate(nodes):
            if nd.op == "concat":
                self.tensor_buf[nd.dst] = buf_of[nd.dst]
                continue
            st = storage(nd.dst)
            if st not in buf_of:
                if free:
                    buf_of[st] = free.pop()
                else:
                    buf_of[st] = n_bufs
                    n_bufs += 1
            L = gpulet.Layer()
            L.in_buf, L.out_buf, L.res_buf = buf_of[storage(nd.src)], buf_of[st], -1
            if nd.op == "conv" and "dst2" in nd.attr:      # the second output has a buffer of its own
                if free:
                    buf_of[nd.attr["dst2"]] = free.pop()
                else:
                    buf_of[nd.attr["dst2"]] = n_bufs
                    n_bufs += 1
                L.K2, L.out2_buf = nd.attr["K2"], buf_of[nd.attr["dst2"]]
                self.tensor_buf[nd.attr["dst2"]] = L.out2_buf
            if nd.op == "conv" and "pool_dst" in nd.attr:  # and so has the pooled input
                if free:
                    buf_of[nd.attr["pool_dst"]] = free.pop()
                else:
                    buf_of[nd.attr["pool_dst"]] = n_bufs
                    n_bufs += 1
                L.side_pool, L.pool_buf = 3, buf_of[nd.attr["pool_dst"]]
                self.tensor_buf[nd.attr["pool_dst"]] = L.pool_buf
            if storage(nd.src) != nd.src:
                raise ValueError("reading a concat slice on its own is not supported")
            a = nd.attr
            if nd.op == "conv":
                if "parts" in a:
                    w = np.concatenate([np.asarray(params[n][0]) for n in a["parts"]], axis=0)
                    b = np.concatenate([np.asarray(params[n][1]) for n in a["parts"]], axis=0)
                else:
                    w, b = params[nd.name]
                C, K = a["C"], a["K"]
                if nd.src == "x" and self.in_pad:
                    w = np.pad(np.asarray(w), ((0, 0), (0, self.in_pad), (0, 0), (0, 0)))
                    C += self.in_pad
                if c_extra.get(nd.src):          # the input carries zero channels: zero weights for them
                    w = np.pad(np.asarray(w), ((0, 0), (0, c_extra[nd.src]), (0, 0), (0, 0)))
                    C += c_extra[nd.src]
                if self.k_pad.get(nd.name):      # zero filters (and zero bias) up to a multiple of 8
                    w = np.pad(np.asarray(w), ((0, self.k_pad[nd.name]), (0, 0), (0, 0), (0, 0)))
                    b = np.pad(np.asarray(b), (0, self.k_pad[nd.name]))
                    K += self.k_pad[nd.name]
                wd = kcrs_to_krsc(w, self.device)
                bd = torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).to(self.device)
                self._keep += [wd, bd]
                L.op, L.C, L.K, L.R, L.S = gpulet.OP_CONV, C, K, a["k"], a["k"]
                L.stride, L.pad, L.relu = a["stride"], a["pad"], int(a["relu"])
                L.pre_pool = a.get("pre_pool", 0)
                L.group_next = a.get("group_next", 0)
                if "in_slice" in a:
                    L.in_ch_offset, L.in_ch_total = a["in_slice"]
                if a["residual"]:
                    L.res_buf = buf_of[storage(a["residual"])]
                if nd.dst in alias:
                    _, off, total = alias[nd.dst]
                    L.out_ch_total, L.out_ch_offset = total, off
                L.w, L.b = wd.data_ptr(), bd.data_ptr()
            elif nd.op == "dwconv":
                w, b = params[nd.name]
                wd = to_device_bf16(np.transpose(np.asarray(w)[:, 0], (1, 2, 0)), self.device)   # (C,1,R,S) -> RSC
                bd = torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).to(self.device)
                self._keep += [wd, bd]
                L.op, L.C, L.R, L.S = gpulet.OP_DWCONV, a["C"], a["k"], a["k"]
                L.stride, L.pad, L.relu = a["stride"], a["pad"], int(a["relu"])
                L.w, L.b = wd.data_ptr(), bd.data_ptr()
            elif nd.op == "maxpool":
                L.op, L.C, L.R, L.stride, L.pad = gpulet.OP_POOL, chans[nd.src], a["k"], a["stride"], a["pad"]
                L.mode = gpulet.POOL_MAX
            elif nd.op == "gavgpool":
                L.op, L.C, L.R, L.stride, L.mode = gpulet.OP_POOL, chans[nd.src], 1, 1, gpulet.POOL_GLOBAL_AVG
            elif nd.op == "fc":
                w, b = params[nd.name]
                C = chans[nd.src]
                hw = a["In"] // C
                if producers.get(nd.src) is not None and producers[nd.src].op != "fc" and hw > 1:
                    w = np.asarray(w).reshape(a["Out"], C, hw).transpose(0, 2, 1).reshape(a["Out"], a["In"])
                wd = to_device_bf16(w, self.device)
                bd = torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).to(self.device)
                self._keep += [wd, bd]
                L.op, L.C, L.K, L.relu = gpulet.OP_FC, a["In"], a["Out"], int(a["relu"])
                L.out_fp32 = int(nd.dst == model.out)
                L.w, L.b = wd.data_ptr(), bd.data_ptr()
            else:
                raise ValueError("unknown node kind %r" % (nd.op,))
            layers.append(L)
            self.tensor_buf[nd.dst] = buf_of[st]
            # release buffers whose last reader was this node (never the input or output); inside a
            # launch group only after its last member, whose launch is also the other members'
            if nd.op == "conv" and nd.attr.get("group_next"):
                continue
            for t, last in list(last_use.items()):
                if reuse and last <= i and t in buf_of and buf_of[t] > 1:
                    free.append(buf_of.pop(t))
                    del last_use[t]

        self.layers = (gpulet.Layer * len(layers))(*layers)
        d = gpulet.ModelDesc()
        d.n_layers, d.n_bufs = len(layers), n_bufs
        d.in_C, d.in_H, d.in_W = self.in_shape[0] + self.in_pad, self.in_shape[1], self.in_shape[2]
        d.in_buf, d.out_buf = 0, 1
        d.layers = self.layers
        self.desc = d
        self.out_fp32 = producers[model.out].op == "fc"
        self._ws = {}

    def _stack_siblings(self, nodes, chans, alias, model):
        """With ``merge_siblings`` convolutions that read the same tensor run as ONE convolution over
        their concatenated filters where the result can be used in place:
          * convolutions of equal geometry that store into adjacent slices of the same
            concatenated tensor (the box and class heads of an SSD feature map): the merged
            layer stores the combined slice;
          * plain 1x1 convolutions that feed only other convolutions (the two reduce layers of an
            inception block): each consumer reads its channel slice of the merged result;
          * with those, one 1x1 convolution of the same tensor that stores into a concatenated
            tensor (the block's 1x1 branch): its filters come first and go to the concatenated
            tensor, the others to the second output of the same launch.
        Every output element is the same sum in the same order, so the bits do not change;
        ``merged`` lists the groups.
        """
        readers = {}
        for nd in nodes:
            reads = list(nd.src) if nd.op == "concat" else [nd.src]
            if nd.op == "conv" and nd.attr["residual"]:
                reads.append(nd.attr["residual"])
            for t in reads:
                readers.setdefault(t, []).append(nd)
        index = {nd.name: i for i, nd in enumerate(nodes)}
        sliced, stored = {}, {}
        for nd in nodes:
            a = nd.attr
            if nd.op != "conv" or a["residual"] or a.get("pre_pool") or nd.src == "x" or nd.dst == model.out:
                continue
            rs = readers.get(nd.dst, [])
            geom = (a["k"], a["stride"], a["pad"], bool(a["relu"]))
            if nd.dst in alias:
                if len(rs) == 1 and rs[0].op == "concat":
                    stored.setdefault((nd.src, alias[nd.dst][0]) + geom, []).append(nd)
            elif (geom[:3] == (1, 1, 0) and a["K"] % 8 == 0 and rs
                  and all(r.op == "conv" and r.src == nd.dst and r.attr["residual"] != nd.dst for r in rs)):
                sliced.setdefault((nd.src,) + geom, []).append(nd)
        in_slice, first, dropped, renamed = {}, {}, set(), {}

        def merge(g, lead=None):
            parts = ([lead] if lead else []) + g
            name = "+".join(n.name for n in g)          # the tensor that holds the outputs of g
            attr = dict(parts[0].attr, K=sum(n.attr["K"] for n in parts), parts=[n.name for n in parts])
            if lead:
                attr.update(K2=sum(n.attr["K"] for n in g), dst2=name)
                node = lead._replace(name="+".join(n.name for n in parts), attr=attr)
            else:
                node = g[0]._replace(name=name, dst=name, attr=attr)
            first[min(parts, key=lambda n: index[n.name]).name] = node
            dropped.update(n.name for n in parts)
            chans[name] = sum(n.attr["K"] for n in g)
            self.merged.append([n.name for n in parts])
            return name

        for g in stored.values():
            g.sort(key=lambda n: alias[n.dst][1])
            runs = [[g[0]]]
            for n in g[1:]:
                last = runs[-1][-1]
                if alias[n.dst][1] == alias[last.dst][1] + last.attr["K"]:
                    runs[-1].append(n)
                else:
                    runs.append([n])
            for run in runs:
                if len(run) >= 2:
                    cat, off, total = alias[run[0].dst]
                    name = merge(run)
                    for n in run:
                        del alias[n.dst]
                        renamed[n.dst] = None
                    renamed[run[0].dst] = name
                    alias[name] = (cat, off, total)
        for key, g in sliced.items():
            lead = None
            if chans[key[0]] % 8 == 0:
                for k2, cand in stored.items():
                    if k2[0] == key[0] and k2[2:] == key[1:]:
                        for n in cand:
                            if (n.name not in dropped and n.attr["K"] % 8 == 0 and alias[n.dst][1] % 8 == 0
                                    and alias[n.dst][2] % 8 == 0 and lead is None):
                                lead = n
            if len(g) + (lead is not None) >= 2:
                name, off = merge(g, lead), 0
                for n in g:
                    in_slice[n.dst] = (name, off, chans[name])
                    off += n.attr["K"]
        kept = []
        for nd in nodes:
            if nd.name in first:
                kept.append(first[nd.name])
            elif nd.name in dropped:
                continue
            elif nd.op == "conv" and nd.src in in_slice:
                t, off, total = in_slice[nd.src]
                if (off, total) != (0, nd.attr["C"]):
                    nd = nd._replace(attr=dict(nd.attr, in_slice=(off, total)))
                kept.append(nd._replace(src=t))
            elif nd.op == "concat":
                kept.append(nd._replace(src=[renamed.get(t, t) for t in nd.src if renamed.get(t, t) is not None]))
            else:
                kept.append(nd)
        nodes = kept
        return nodes

    def _ride_pools(self, nodes, chans, alias, model):
        # A 3x3 / stride 1 / pad 1 max pool whose input is also read by a plain 1x1 convolution
        # (an inception block's pooling branch next to its 1x1 layers) rides along with that
        # convolution's launch: extra workgroups of the same grid do the pooling.
        hosts, first_read = {}, {}
        for i, nd in enumerate(nodes):
            a = nd.attr
            if (nd.op == "conv" and (a["k"], a["stride"], a["pad"]) == (1, 1, 0) and not a["residual"]
                    and not a.get("pre_pool") and "in_slice" not in a and nd.src != "x"
                    and nd.src not in alias and chans[nd.src] % 8 == 0):
                hosts.setdefault(nd.src, (i, nd.name))
            for t in (list(nd.src) if nd.op == "concat" else [nd.src]):
                first_read.setdefault(t, i)
        riders, kept = {}, []
        for i, nd in enumerate(nodes):
            a = nd.attr
            if (nd.op == "maxpool" and (a["k"], a["stride"], a["pad"]) == (3, 1, 1) and nd.dst != model.out
                    and nd.src in hosts and hosts[nd.src][1] not in riders
                    and hosts[nd.src][0] < first_read.get(nd.dst, len(nodes))):
                riders[hosts[nd.src][1]] = nd
                continue
            kept.append(nd)
        nodes = [nd._replace(attr=dict(nd.attr, pool_dst=riders[nd.name].dst)) if nd.name in riders else nd
                 for nd in kept]
        self.side_pools = [r.name for r in riders.values()]
        return nodes

    def _chain_groups(self, nodes, alias):
        # Independent convolutions share a launch (``groups``): a sibling that reads the same
        # tensor is first moved next to its sibling when nothing in between stands in the way (a
        # projection shortcut next to the first layer of its residual block), then runs of
        # adjacent convolutions that neither read nor overwrite one another's tensors are chained.
        def reads_of(nd):
            r = list(nd.src) if nd.op == "concat" else [nd.src]
            if nd.op == "conv" and nd.attr["residual"]:
                r.append(nd.attr["residual"])
            return r

        def shareable(nd):
            a = nd.attr
            return (nd.op == "conv" and a["C"] % 8 == 0 and nd.src != "x" and not a.get("pre_pool")
                    and "dst2" not in a and "pool_dst" not in a)

        def independent(p, q):
            if p.dst in reads_of(q) or q.dst in reads_of(p):
                return False
            sp, sq = storage(p.dst), storage(q.dst)
            return sp != sq or (p.dst in alias and q.dst in alias)

        def storage(t):
            return alias[t][0] if t in alias else t

        i = 0
        while i < len(nodes):
            if shareable(nodes[i]):
                for j in range(i + 2, min(i + 4, len(nodes))):
                    between = nodes[i + 1:j]
                    if (shareable(nodes[j]) and nodes[j].src == nodes[i].src
                            and all(b.op != "concat" and independent(b, nodes[j]) for b in between)):
                        nodes.insert(i + 1, nodes.pop(j))
                        break
            i += 1
        self.groups, run = [], []
        for k, nd in enumerate(nodes + [None]):
            if nd is not None and nd.op == "concat":
                continue            # emits no layer: members on either side of it stay neighbours
            if (nd is not None and shareable(nd) and len(run) < 4
                    and all(independent(nodes[m], nd) for m in run)):
                run.append(k)
                continue
            if len(run) >= 2:
                for m in run[:-1]:
                    nodes[m] = nodes[m]._replace(attr=dict(nodes[m].attr, group_next=1))
                self.groups.append([nodes[m].name for m in run])
            run = [k] if nd is not None and shareable(nd) else []
        return nodes

    def input_to_device(self, x_nchw):
        """Host batch (N, C, H, W) -> device NHWC bf16 with the channel padding the model expects."""
        x = np.asarray(x_nchw)
        if self.in_pad:
            x = np.pad(x, ((0, 0), (0, self.in_pad), (0, 0), (0, 0)))
        return nchw_to_nhwc(x, self.device)

    def output_shape(self, batch):
        C, H, W, _, _ = gpulet.model_buffer_info(self.desc, batch, 1)
        return (batch, H, W, C)

    def workspace(self, batch):
        """Device workspace for ``batch`` images -> (tensor, bytes)."""
        if batch not in self._ws:
            n = gpulet.model_workspace_bytes(self.desc, batch)
            self._ws[batch] = (torch.empty(max(n, 256), dtype=torch.uint8, device=self.device), n)
        return self._ws[batch]

    def alloc_output(self, batch):
        dt = torch.float32 if self.out_fp32 else torch.bfloat16
        return torch.empty(self.output_shape(batch), dtype=dt, device=self.device)

    def run(self, partition, x_nhwc, timed=False):
        """Forward pass of one batch (device NHWC bf16) -> (output tensor, ms or None)."""
        batch = x_nhwc.shape[0]
        ws, n = self.workspace(batch)
        y = self.alloc_output(batch)
        torch.cuda.synchronize(self.device)
        ms = gpulet.run_model(self.desc, batch, partition, x_nhwc, y, ws, n, timed=timed)
        partition.sync()
        return y, ms

    def read_tensor(self, name, batch):
        """Copy of a named intermediate tensor (NHWC) from the workspace after a run.
        Only meaningful for tensors whose buffer was not reused later, and, for the output of a
        convolution that feeds nothing but a 2x2 / stride 2 max pool, only with
        ``gpulet.set_conv_pool_fusion(False)`` (the pair may otherwise run as one launch that never
        writes it)."""
        buf = self.tensor_buf[name]
        ws, _ = self.workspace(batch)
        C, H, W, e, off = gpulet.model_buffer_info(self.desc, batch, buf)
        n = batch * C * H * W * e
        raw = ws[off:off + n]
        return raw.view(torch.bfloat16 if e == 2 else torch.float32).reshape(batch, H, W, C).clone()
