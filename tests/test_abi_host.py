"""Host-side checks that need no GPU: the shared library loads and exports
every symbol the header declares, mask arithmetic and bookkeeping are exact,
argument errors are reported before any GPU call, and the model description
is validated with the shapes the tables imply."""

import ctypes
import os
import re

import numpy as np
import pytest

from paper_2109_01611_amd import gpulet

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gpulet_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 20
    raw = ctypes.CDLL(gpulet.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    assert set(names) == set(gpulet.EXPORTS)


def test_status_strings():
    for s, word in [(0, "OK"), (-1, "EINVAL"), (-2, "EOVERSUB"), (-3, "EHIP"), (-4, "ENOMEM"), (-99, "?")]:
        assert word in gpulet.status_string(s)


def _popcount(words):
    return sum(bin(w).count("1") for w in words)


@pytest.mark.parametrize("pct,n_cu", [(20, 64), (25, 64), (40, 96), (50, 128), (60, 160), (80, 192),
                                      (100, 256), (1, 32), (99, 224), (12, 32), (13, 32), (19, 64)])
def test_mask_sizes_on_256_cus(pct, n_cu):
    words, n = gpulet.mask_for_pct(256, 8, pct, 0)
    assert len(words) == 8 and n == n_cu and _popcount(words) == n_cu
    # the first n/8 CUs of every die are the lowest n bits
    as_int = sum(w << (32 * i) for i, w in enumerate(words))
    assert as_int == (1 << n_cu) - 1


@pytest.mark.parametrize("pct", [1, 20, 25, 33, 40, 50, 60, 75, 80, 99])
def test_split_gives_disjoint_cover(pct):
    a, na = gpulet.mask_for_pct(256, 8, pct, 0)
    b, nb = gpulet.mask_for_pct(256, 8, 100 - pct, 1)
    assert na + nb == 256
    for x, y in zip(a, b):
        assert x & y == 0 and (x | y) == 0xFFFFFFFF
    # per-die symmetry: bit i is CU i // 8 of die i % 8
    bits = [i for i in range(256) if (a[i // 32] >> (i % 32)) & 1]
    per_die = [sum(1 for i in bits if i % 8 == d) for d in range(8)]
    assert len(set(per_die)) == 1
    # ... and CU c of a die is in shader engine c % 4: every engine contributes the same count
    per_engine = [sum(1 for i in bits if i % 8 == 0 and (i // 8) % 4 == e) for e in range(4)]
    assert len(set(per_engine)) == 1 and per_engine[0] >= 1


def test_two_partitions_never_overlap_when_sizes_fit():
    for p in range(1, 100):
        for q in range(1, 101 - p):
            a, _ = gpulet.mask_for_pct(256, 8, p, 0)
            b, _ = gpulet.mask_for_pct(256, 8, q, 1)
            assert all(x & y == 0 for x, y in zip(a, b)), (p, q)


def test_mask_other_geometries_and_errors():
    words, n = gpulet.mask_for_pct(64, 1, 25, 0)
    assert n == 16 and words == [0xFFFF, 0]
    words, n = gpulet.mask_for_pct(64, 1, 75, 1)
    assert n == 48 and words == [0xFFFF0000, 0xFFFFFFFF]
    # dies that cannot be split by shader engine round to whole CUs, at least one on each side
    assert gpulet.mask_for_pct(6, 1, 50, 0) == ([0b000111], 3)
    assert gpulet.mask_for_pct(6, 1, 1, 0) == ([0b000001], 1)
    assert gpulet.mask_for_pct(6, 1, 1, 1) == ([0b000001 << 5], 1)
    assert gpulet.mask_for_pct(30, 3, 40, 0)[1] == 12
    for args in [(256, 8, 0, 0), (256, 8, 101, 0), (256, 8, 50, 2), (255, 8, 50, 0), (0, 8, 50, 0), (256, 0, 50, 0)]:
        with pytest.raises(gpulet.GpuletError) as e:
            gpulet.mask_for_pct(*args)
        assert e.value.status == gpulet.EINVAL
    w = (ctypes.c_uint32 * 8)()
    nw, nc = ctypes.c_int(), ctypes.c_int()
    assert gpulet.lib.gpulet_mask_for_pct(256, 8, 50, 0, w, 4, ctypes.byref(nw), ctypes.byref(nc)) == gpulet.ENOMEM
    assert gpulet.lib.gpulet_mask_for_pct(256, 8, 50, 0, None, 8, ctypes.byref(nw), ctypes.byref(nc)) == gpulet.EINVAL


def test_latency_stats_nearest_rank():
    lat = [float(v) for v in range(1, 201)]          # 1..200
    rng = np.random.default_rng(0)
    rng.shuffle(lat)
    mean, p50, p99 = gpulet.latency_stats(lat)
    assert mean == 100.5 and p50 == 100.0 and p99 == 198.0   # ceil(0.99*200) = 198
    assert gpulet.latency_stats([3.0]) == (3.0, 3.0, 3.0)
    assert gpulet.latency_stats([1.0, 2.0])[1:] == (1.0, 2.0)
    with pytest.raises(gpulet.GpuletError):
        gpulet.latency_stats([])


def test_layer_calls_reject_bad_arguments_before_touching_the_gpu():
    x = w = y = 4096  # stand-in non-NULL addresses; never dereferenced on these paths
    ok = dict(N=1, C=8, H=8, W=8, K=8, R=3, S=3, stride=1, pad=1, relu=1)
    bad = [dict(ok, N=0), dict(ok, C=-1), dict(ok, stride=0), dict(ok, pad=-1), dict(ok, R=0),
           dict(ok, H=2, pad=0, R=5, S=5),                 # empty output
           dict(ok, N=1 << 20, H=64, W=64, C=64)]          # 2^38 elements
    for kw in bad:
        with pytest.raises(gpulet.GpuletError) as e:
            gpulet.conv2d_fwd(x, w, None, y, **kw)
        assert e.value.status == gpulet.EINVAL, kw
    for args in [(None, w, None, y), (x, None, None, y), (x, w, None, None)]:
        with pytest.raises(gpulet.GpuletError):
            gpulet.conv2d_fwd(*args, **ok)
    with pytest.raises(gpulet.GpuletError):   # slice does not fit the destination
        gpulet.conv2d_fwd_ex(x, w, None, y, residual=None, y_ch_stride=12, y_ch_offset=8, **ok)
    for xs, xo in ((12, 8), (16, -8), (4, 0)):   # slice does not fit the source pixels
        with pytest.raises(gpulet.GpuletError) as e:
            gpulet.conv2d_fwd_slices(x, w, None, y, residual=None, x_ch_stride=xs, x_ch_offset=xo, **ok)
        assert e.value.status == gpulet.EINVAL
    # launch groups: members must not depend on one another
    m0 = dict(x=1 << 20, w=w, y=2 << 20, **ok)
    for m1 in (dict(x=2 << 20, w=w, y=3 << 20, **ok),                    # reads what the other writes
               dict(x=1 << 20, w=w, y=2 << 20, **ok),                    # writes the same tensor
               dict(x=1 << 20, w=w, y=3 << 20, residual=(2 << 20) + 64, **ok),
               dict(x=1 << 20, w=w, y=(2 << 20) - 64, **ok),             # outputs overlap
               dict(x=1 << 20, w=w, y=2 << 20, y_ch_stride=16, y_ch_offset=4, **ok)):  # slices of different tensors
        with pytest.raises(gpulet.GpuletError) as e:
            gpulet.conv2d_group_fwd([m0, m1])
        assert e.value.status == gpulet.EINVAL, m1
    with pytest.raises(gpulet.GpuletError) as e:
        gpulet.conv2d_group_fwd([m0] * 5)
    assert e.value.status == gpulet.EINVAL
    with pytest.raises(gpulet.GpuletError) as e:
        gpulet.conv2d_group_fwd([m0, dict(m0, y=3 << 20, C=0)])
    assert e.value.status == gpulet.EINVAL
    with pytest.raises(gpulet.GpuletError):
        gpulet.pool(x, y, 1, 8, 8, 8, gpulet.POOL_MAX, k=2, stride=2, pad=2)    # pad >= k
    with pytest.raises(gpulet.GpuletError):
        gpulet.pool(x, y, 1, 8, 8, 8, 7, k=2, stride=2, pad=0)                  # unknown mode
    with pytest.raises(gpulet.GpuletError):
        gpulet.pool(None, y, 1, 8, 8, 8, gpulet.POOL_MAX, k=2, stride=2, pad=0)
    with pytest.raises(gpulet.GpuletError):
        gpulet.fc(x, w, None, y, 0, 8, 8, relu=0)
    with pytest.raises(gpulet.GpuletError):
        gpulet.fc(x, w, None, y, 1 << 16, 1 << 16, 8, relu=0)
    with pytest.raises(gpulet.GpuletError) as e:
        gpulet.Partition(0, 0)
    assert e.value.status == gpulet.EINVAL
    with pytest.raises(gpulet.GpuletError) as e:
        gpulet.Partition(0, 50, which=3)
    assert e.value.status == gpulet.EINVAL
    assert gpulet.lib.gpulet_partition_destroy(None) == gpulet.EINVAL
    assert gpulet.lib.gpulet_partition_destroy(ctypes.c_void_p(12345)) == gpulet.EINVAL


def _layer(**kw):
    L = gpulet.Layer()
    L.res_buf = -1
    for k, v in kw.items():
        setattr(L, k, v)
    return L


def _desc(layers, n_bufs, in_shape, in_buf=0, out_buf=1):
    arr = (gpulet.Layer * len(layers))(*layers)
    d = gpulet.ModelDesc()
    d.n_layers, d.n_bufs = len(layers), n_bufs
    d.in_C, d.in_H, d.in_W = in_shape
    d.in_buf, d.out_buf = in_buf, out_buf
    d.layers = arr
    d._arr = arr
    return d


def test_model_shape_inference_and_workspace_layout():
    W = 4096  # stand-in weight address
    layers = [
        _layer(op=gpulet.OP_CONV, in_buf=0, out_buf=2, C=3, K=16, R=7, S=7, stride=2, pad=3, relu=1, w=W),
        _layer(op=gpulet.OP_POOL, in_buf=2, out_buf=3, C=16, R=3, stride=2, pad=1, mode=gpulet.POOL_MAX),
        # two branches concatenated into buffer 4 (8 + 24 channels)
        _layer(op=gpulet.OP_CONV, in_buf=3, out_buf=4, C=16, K=8, R=1, S=1, stride=1, pad=0, relu=1, w=W,
               out_ch_total=32, out_ch_offset=0),
        _layer(op=gpulet.OP_CONV, in_buf=3, out_buf=4, C=16, K=24, R=3, S=3, stride=1, pad=1, relu=1, w=W,
               out_ch_total=32, out_ch_offset=8),
        _layer(op=gpulet.OP_CONV, in_buf=4, out_buf=2, C=32, K=32, R=1, S=1, stride=1, pad=0, relu=1, w=W,
               res_buf=4),
        _layer(op=gpulet.OP_POOL, in_buf=2, out_buf=3, C=32, R=1, stride=1, mode=gpulet.POOL_GLOBAL_AVG),
        _layer(op=gpulet.OP_FC, in_buf=3, out_buf=1, C=32, K=10, out_fp32=1, w=W),
    ]
    d = _desc(layers, 5, (3, 64, 64))
    batch = 4
    # buffer 2: conv out 16x32x32 (32 KiB/img in bf16), later 32x16x16 (16 KiB) -> 32 KiB
    # buffer 3: pool out 16x16x16 (8 KiB), later 32x1x1 -> 8 KiB;  buffer 4: 32x16x16 -> 16 KiB
    assert gpulet.model_workspace_bytes(d, batch) == batch * (32768 + 8192 + 16384)
    assert gpulet.model_buffer_info(d, batch, 4) == (32, 16, 16, 2, batch * (32768 + 8192))
    assert gpulet.model_buffer_info(d, batch, 2) == (32, 16, 16, 2, 0)
    assert gpulet.model_buffer_info(d, batch, 1) == (10, 1, 1, 4, None)
    assert gpulet.model_buffer_info(d, batch, 0) == (3, 64, 64, 2, None)
    # odd sizes round every buffer up to 256 bytes
    d1 = _desc([_layer(op=gpulet.OP_CONV, in_buf=0, out_buf=2, C=1, K=3, R=3, S=3, stride=1, pad=0, w=W),
                _layer(op=gpulet.OP_POOL, in_buf=2, out_buf=1, C=3, R=1, stride=1, mode=gpulet.POOL_GLOBAL_AVG)],
               3, (1, 5, 5))
    assert gpulet.model_workspace_bytes(d1, 1) == 256       # 3*3*3*2 = 54 bytes -> 256


def test_model_description_errors():
    W = 4096
    good = _layer(op=gpulet.OP_CONV, in_buf=0, out_buf=1, C=3, K=8, R=3, S=3, stride=1, pad=1, w=W)
    assert gpulet.model_workspace_bytes(_desc([good], 2, (3, 8, 8)), 2) == 0

    def bad(layers, n_bufs=3, in_shape=(3, 8, 8), batch=1, **kw):
        with pytest.raises(gpulet.GpuletError) as e:
            gpulet.model_workspace_bytes(_desc(layers, n_bufs, in_shape, **kw), batch)
        assert e.value.status == gpulet.EINVAL
    bad([_layer(op=gpulet.OP_CONV, in_buf=0, out_buf=1, C=4, K=8, R=3, S=3, stride=1, pad=1, w=W)])  # C mismatch
    bad([_layer(op=gpulet.OP_CONV, in_buf=2, out_buf=1, C=3, K=8, R=3, S=3, stride=1, pad=1, w=W)])  # read before write
    bad([_layer(op=gpulet.OP_CONV, in_buf=0, out_buf=0, C=3, K=8, R=3, S=3, stride=1, pad=1, w=W)])  # writes the input
    bad([_layer(op=gpulet.OP_CONV, in_buf=0, out_buf=5, C=3, K=8, R=3, S=3, stride=1, pad=1, w=W)])  # bad index
    bad([_layer(op=gpulet.OP_CONV, in_buf=0, out_buf=1, C=3, K=8, R=3, S=3, stride=1, pad=1, w=None)])  # no weights
    bad([_layer(op=gpulet.OP_CONV, in_buf=0, out_buf=2, C=3, K=8, R=3, S=3, stride=1, pad=1, w=W)])  # output never written
    bad([_layer(op=gpulet.OP_CONV, in_buf=0, out_buf=1, C=3, K=8, R=9, S=9, stride=1, pad=0, w=W)], in_shape=(3, 8, 8))
    bad([_layer(op=gpulet.OP_FC, in_buf=0, out_buf=1, C=100, K=8, w=W)])                             # In != C*H*W
    bad([_layer(op=9, in_buf=0, out_buf=1)])
    bad([good], batch=0)
    bad([good], in_buf=1, out_buf=1)
    bad([_layer(op=gpulet.OP_CONV, in_buf=0, out_buf=1, C=3, K=8, R=3, S=3, stride=1, pad=1, w=W, res_buf=2)])
    # a layer reading a channel slice: the stated pixel width must be the source's, the slice inside it
    reduce_ = _layer(op=gpulet.OP_CONV, in_buf=0, out_buf=2, C=3, K=24, R=1, S=1, stride=1, pad=0, w=W)
    take = dict(op=gpulet.OP_CONV, in_buf=2, out_buf=1, C=8, K=8, R=3, S=3, stride=1, pad=1, w=W)
    assert gpulet.model_workspace_bytes(_desc([reduce_, _layer(in_ch_total=24, in_ch_offset=16, **take)], 3,
                                              (3, 8, 8)), 2) == 2 * 24 * 8 * 8 * 2
    bad([reduce_, _layer(**take)])
    bad([reduce_, _layer(in_ch_total=32, in_ch_offset=16, **take)])
    bad([reduce_, _layer(in_ch_total=24, in_ch_offset=17, **take)])
    bad([reduce_, _layer(in_ch_total=24, in_ch_offset=-1, **take)])
    # a layer with two outputs: 1x1 only, no residual, a second buffer of its own, 0 < K2 < K
    two = dict(op=gpulet.OP_CONV, in_buf=0, out_buf=2, C=3, K=24, R=1, S=1, stride=1, pad=0, w=W)
    use = [_layer(op=gpulet.OP_CONV, in_buf=3, out_buf=1, C=16, K=8, R=3, S=3, stride=1, pad=1, w=W)]
    assert gpulet.model_workspace_bytes(_desc([_layer(K2=16, out2_buf=3, **two)] + use, 4, (3, 8, 8)), 2) == \
        2 * (8 + 16) * 8 * 8 * 2
    assert gpulet.model_buffer_info(_desc([_layer(K2=16, out2_buf=3, **two)] + use, 4, (3, 8, 8)), 2, 2)[:3] == (8, 8, 8)
    bad([_layer(K2=24, out2_buf=3, **two)] + use, n_bufs=4)
    bad([_layer(K2=-1, out2_buf=3, **two)] + use, n_bufs=4)
    bad([_layer(K2=16, out2_buf=2, **two)] + use, n_bufs=4)          # both parts to one buffer
    bad([_layer(K2=16, out2_buf=0, **two)] + use, n_bufs=4)          # the model input
    bad([_layer(K2=16, out2_buf=4, **two)] + use, n_bufs=4)          # bad index
    bad([_layer(K2=16, out2_buf=3, out2_ch_total=8, **two)] + use, n_bufs=4)   # slice does not fit
    bad([_layer(K2=16, out2_buf=3, **dict(two, R=3, S=3, pad=1))] + use, n_bufs=4)
    # a 1x1 layer that carries the max pool of its input: a buffer of its own, window 3 only, dense input
    rider = dict(op=gpulet.OP_CONV, in_buf=2, out_buf=3, C=8, K=8, R=1, S=1, stride=1, pad=0, w=W)
    head = [_layer(op=gpulet.OP_CONV, in_buf=0, out_buf=2, C=3, K=8, R=3, S=3, stride=1, pad=1, w=W)]
    tail = [_layer(op=gpulet.OP_CONV, in_buf=4, out_buf=1, C=8, K=8, R=1, S=1, stride=1, pad=0, w=W, res_buf=3)]
    d = _desc(head + [_layer(side_pool=3, pool_buf=4, **rider)] + tail, 5, (3, 8, 8))
    assert gpulet.model_workspace_bytes(d, 2) == 3 * 2 * 8 * 8 * 8 * 2
    assert gpulet.model_buffer_info(d, 2, 4)[:4] == (8, 8, 8, 2)
    bad(head + [_layer(side_pool=2, pool_buf=4, **rider)] + tail, n_bufs=5)
    bad(head + [_layer(side_pool=3, pool_buf=3, **rider)] + tail, n_bufs=5)      # the layer's own output
    bad(head + [_layer(side_pool=3, pool_buf=2, **rider)] + tail, n_bufs=5)      # its input
    bad(head + [_layer(side_pool=3, pool_buf=5, **rider)] + tail, n_bufs=5)
    bad(head + [_layer(side_pool=3, pool_buf=4, **dict(rider, R=3, S=3, pad=1))] + tail, n_bufs=5)
    bad(head + [_layer(**rider)] + tail, n_bufs=5)                               # buffer 4 never written
    # launch groups: convolutions only, independent of one another, at most four, inside the table
    g0 = dict(op=gpulet.OP_CONV, in_buf=0, C=3, K=8, R=3, S=3, stride=1, pad=1, w=W)
    fin = [_layer(op=gpulet.OP_CONV, in_buf=2, out_buf=1, C=8, K=8, R=1, S=1, stride=1, pad=0, w=W, res_buf=3)]
    assert gpulet.model_workspace_bytes(
        _desc([_layer(out_buf=2, group_next=1, **g0), _layer(out_buf=3, **g0)] + fin, 4, (3, 8, 8)), 1) == 2 * 8 * 8 * 8 * 2
    bad([_layer(out_buf=2, group_next=1, **g0), _layer(out_buf=2, **g0)] + fin, n_bufs=4)     # same destination
    bad([_layer(out_buf=2, group_next=1, **g0),
         _layer(op=gpulet.OP_CONV, in_buf=2, out_buf=3, C=8, K=8, R=1, S=1, stride=1, pad=0, w=W)] + fin, n_bufs=4)
    bad([_layer(out_buf=2, group_next=1, **g0), _layer(op=gpulet.OP_POOL, in_buf=0, out_buf=3, C=3, R=3, stride=1,
                                                       pad=1, mode=gpulet.POOL_MAX)], n_bufs=4)
    bad([_layer(out_buf=2, **g0), _layer(out_buf=3, **g0),                                    # chain runs off the table
         _layer(op=gpulet.OP_CONV, in_buf=2, out_buf=1, C=8, K=8, R=1, S=1, stride=1, pad=0, w=W, res_buf=3,
                group_next=1)], n_bufs=4)
    bad([_layer(out_buf=b, group_next=1, **g0) for b in (2, 3, 4, 5)] + [_layer(out_buf=6, **g0)] + fin, n_bufs=7)
    # two slices of one tensor are fine, overlapping ones are not
    cat = [_layer(op=gpulet.OP_CONV, in_buf=2, out_buf=1, C=16, K=8, R=1, S=1, stride=1, pad=0, w=W)]
    assert gpulet.model_workspace_bytes(
        _desc([_layer(out_buf=2, out_ch_total=16, out_ch_offset=0, group_next=1, **g0),
               _layer(out_buf=2, out_ch_total=16, out_ch_offset=8, **g0)] + cat, 3, (3, 8, 8)), 1) == 16 * 8 * 8 * 2
    bad([_layer(out_buf=2, out_ch_total=16, out_ch_offset=0, group_next=1, **g0),
         _layer(out_buf=2, out_ch_total=16, out_ch_offset=4, **g0)] + cat)
    # residual of the wrong shape
    bad([_layer(op=gpulet.OP_CONV, in_buf=0, out_buf=2, C=3, K=8, R=3, S=3, stride=2, pad=1, w=W),
         _layer(op=gpulet.OP_CONV, in_buf=0, out_buf=1, C=3, K=8, R=3, S=3, stride=1, pad=1, w=W, res_buf=2)])


def test_binding_mirrors_the_header_tile_count():
    import re
    header = open(os.path.join(os.path.dirname(__file__), "..", "include", "gpulet.h")).read()
    m = re.search(r"enum\s*\{\s*GPULET_CONV_TILES\s*=\s*(\d+)\s*\}", header)
    assert m and int(m.group(1)) == gpulet.CONV_TILES
