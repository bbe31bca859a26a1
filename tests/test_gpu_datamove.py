"""GPU parity, pure data movement and the elementwise consumer (bit-exact bar)."""
import numpy as np
import pytest

import workloads
from oracle import consumers, dm_ops, index_maps
from oracle.run import run_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2604_09558_amd as vt
    from paper_2604_09558_amd import torch_io
    vt.lib()
    return vt, torch_io, torch


def bits(a):
    a = np.ascontiguousarray(a)
    return a.view({2: np.uint16, 4: np.uint32}[a.dtype.itemsize])


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_materialize_random_chains_bit_exact(gpu, dtype):
    vt, tio, torch = gpu
    done = 0
    for seed in range(120):
        wl = workloads.random_chain(seed, n_ops=6, dtype=dtype)
        dense = dm_ops.run_chain(wl.chain, wl.sources, wl.index_tables)["R"]
        dw = tio.DeviceWorkload(wl)
        try:
            d = dw.build("R")
        except vt.VtError as e:
            assert e.code == vt.ERR_UNSUPPORTED
            continue
        out = dw.empty(dense.shape)
        out.fill_(-7.0)
        try:
            vt.vt_materialize(d, out)
        except vt.VtError as e:
            assert e.code == vt.ERR_UNSUPPORTED, str(e)
            continue
        torch.cuda.synchronize()
        got = tio.to_host_bits(out)
        assert np.array_equal(bits(got), bits(dense)), (seed, d.dump())
        done += 1
    assert done >= 105, done


def test_materialize_vector_paths_and_ragged(gpu):
    """Larger tensors that take the 16/8/4/2-byte vector paths, several blocks and a ragged tail."""
    vt, tio, torch = gpu
    rng = np.random.default_rng(0)
    cases = [
        # (source shape, chain, result)
        ((6, 40, 8, 64), [("p", "permute", ("X",), {"perm": (0, 2, 1, 3)}), ("R", "reshape", ("p",), {"shape": (48, 2560)})]),
        ((37, 1000), [("R", "slice", ("X",), {"dim": 1, "start": 8, "stop": 1000, "step": 1})]),       # run 992
        ((37, 1001), [("R", "slice", ("X",), {"dim": 1, "start": 3, "stop": 1001, "step": 1})]),       # odd base: scalar path
        ((5, 3, 130), [("u", "unsqueeze", ("X",), {"dim": 1}), ("e", "expand", ("u",), {"shape": (5, 4, 3, 130)}),
                       ("R", "reshape", ("e",), {"shape": (20, 390)})]),
        ((300, 257), [("R", "permute", ("X",), {"perm": (1, 0)})]),
        ((64, 4, 36), [("R", "slice", ("X",), {"dim": 2, "start": 4, "stop": 36, "step": 2})]),
    ]
    for dtype in ("f32", "bf16"):
        for shape, chain in cases:
            x = workloads.encode(rng.normal(size=shape).astype(np.float32), dtype)
            wl = workloads.Workload("case", dtype, {"X": x}, chain, {"kind": "materialize", "x": "R"})
            dense = dm_ops.run_chain(chain, wl.sources)["R"]
            dw = tio.DeviceWorkload(wl)
            d = dw.build("R")
            out = dw.empty(dense.shape)
            vt.vt_materialize(d, out)
            torch.cuda.synchronize()
            assert np.array_equal(bits(tio.to_host_bits(out)), bits(dense)), (dtype, shape, d.dump())


def test_copy_op_each_operator(gpu):
    vt, tio, torch = gpu
    rng = np.random.default_rng(1)
    tables = {"t": np.array([3, 0, 0, 2, 1, 3, 2], np.int32)}
    cases = [
        ("permute", [(6, 5, 16)], {"perm": (2, 0, 1)}),
        ("reshape", [(6, 5, 16)], {"shape": (30, 16)}),
        ("slice", [(9, 64)], {"dim": 1, "start": 8, "stop": 40, "step": 1}),
        ("split", [(9, 64)], {"dim": 1, "sizes": (16, 40, 8), "output": 1}),
        ("concat", [(4, 8), (4, 24), (4, 3)], {"dim": 1}),
        ("unsqueeze", [(4, 8)], {"dim": 1}),
        ("expand", [(4, 1, 8)], {"shape": (4, 5, 8)}),
        ("index_select", [(4, 32)], {"dim": 0, "index": "t"}),
    ]
    for dtype in ("f32", "f16"):
        for op, shapes, p in cases:
            ins = [workloads.encode(rng.normal(size=s).astype(np.float32), dtype) for s in shapes]
            dense = dm_ops.run_statement(op, ins, p, tables)
            brute = index_maps.materialize_bruteforce(op, ins, p, tables)
            assert np.array_equal(bits(dense), bits(brute))
            dev = [tio.to_device(a, dtype) for a in ins]
            tdev = {k: torch.from_numpy(v).cuda() for k, v in tables.items()}
            out = torch.empty(dense.shape, dtype=tio.TORCH_DTYPE[dtype], device="cuda:0")
            vt.vt_copy_op(op, [(a.shape, dtype, t.data_ptr()) for a, t in zip(ins, dev)], p, out,
                          tables=tables, table_ptrs={k: v.data_ptr() for k, v in tdev.items()})
            torch.cuda.synchronize()
            assert np.array_equal(bits(tio.to_host_bits(out)), bits(dense)), (dtype, op)


def run_c1(vt, tio, torch, wl):
    dw = tio.DeviceWorkload(wl)
    v = dw.build("V")
    z = dw.build("Z")
    rows = v.shape[0]
    out = torch.full((rows,), -1.0, dtype=torch.float32, device="cuda:0")
    vt.vt_elementwise(vt.EW_ADD_ROWSUM, v, z, 0.0, out)
    torch.cuda.synchronize()
    return dw, v, z, out


def test_c1_tiny_chain_bit_exact_and_equals_materialized(gpu):
    vt, tio, torch = gpu
    wl = workloads.c1_tiny_chain()
    ref = run_workload(wl, keep_intermediates=True)
    dw, v, z, out = run_c1(vt, tio, torch, wl)
    got = out.cpu().numpy()
    assert np.array_equal(bits(got), bits(ref["out"])), (got, ref["out"])
    assert np.max(np.abs(got.astype(np.float64) - ref["out_f64"])) <= 1e-5
    # materialized path on the GPU: every operator as an explicit copy kernel, then the same consumer
    cur = {k: t for k, t in dw.tensors.items()}
    shapes = {k: tuple(t.shape) for k, t in dw.tensors.items()}
    for name, op, ins, p in wl.chain:
        dense = ref["env"][name]
        o = torch.empty(dense.shape, dtype=torch.float32, device="cuda:0")
        vt.vt_copy_op(op, [(shapes[i], "f32", cur[i].data_ptr()) for i in ins], p, o)
        cur[name], shapes[name] = o, dense.shape
        torch.cuda.synchronize()
        assert np.array_equal(bits(o.cpu().numpy()), bits(dense)), name
    vm = vt.build_chain([], {"V": (shapes["V"], "f32", cur["V"].data_ptr())}, "V")
    out2 = torch.empty(8, dtype=torch.float32, device="cuda:0")
    vt.vt_elementwise(vt.EW_ADD_ROWSUM, vm, z, 0.0, out2)
    torch.cuda.synchronize()
    assert np.array_equal(bits(out2.cpu().numpy()), bits(got))


@pytest.mark.parametrize("sizes", [(3, 5, 7, 1, 12, 4), (30, 50, 130, 7, 1400, 77), (2, 3, 64, 0, 6, 1)])
def test_c1_other_sizes_and_order_pin(gpu, sizes):
    """Rows longer than one wave pass (several columns per lane), ragged widths."""
    vt, tio, torch = gpu
    a, b, c, lo, hi, ny = sizes
    wl = workloads.c1_tiny_chain(seed=3, a=a, b=b, c=c, lo=lo, hi=hi, ny=ny)
    ref = run_workload(wl)
    _, _, _, out = run_c1(vt, tio, torch, wl)
    assert np.array_equal(bits(out.cpu().numpy()), bits(ref["out"]))


def test_rowsum_order_pin_on_gpu(gpu):
    """The cancellation example that separates the fixed order from a sequential sum."""
    vt, tio, torch = gpu
    v = np.zeros((2, 66), np.float32)
    v[0, 0], v[0, 64], v[0, 1], v[0, 65] = 1e8, -1e8, 1.0, 1.0
    v[1, 0], v[1, 1], v[1, 2] = 1e8, 1.0, -1e8
    z = np.zeros_like(v)
    ref = consumers.add_rowsum_f32(v, z)
    assert list(ref) == [2.0, 1.0]
    tv, tz = tio.to_device(v, "f32"), tio.to_device(z, "f32")
    dv = vt.build_chain([], {"V": (v.shape, "f32", tv.data_ptr())}, "V")
    dz = vt.build_chain([], {"Z": (z.shape, "f32", tz.data_ptr())}, "Z")
    out = torch.empty(2, dtype=torch.float32, device="cuda:0")
    vt.vt_elementwise(vt.EW_ADD_ROWSUM, dv, dz, 0.0, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), ref)


@pytest.mark.parametrize("dtype,C,R,cut", [
    ("f16", 128, 6, 0), ("bf16", 96, 6, 0), ("f32", 200, 6, 0), ("f16", 1024, 6, 0), ("f16", 130, 6, 0),
    # more than one wave's 64 rows and a ragged last wave (243 rows); two and four vectors per lane
    ("f16", 128, 9, 0), ("bf16", 1024, 9, 0), ("f16", 2048, 9, 0), ("f32", 512, 9, 0), ("f32", 1024, 9, 0),
    # the last dim sliced: rows are no longer whole contiguous ranges as far as the map's run says,
    # or are contiguous but start off the vector grid
    ("f16", 128, 9, 8), ("f32", 200, 9, 4), ("bf16", 96, 9, 3),
])
def test_layernorm_virtual_rows(gpu, dtype, C, R, cut):
    """LayerNorm over window-partitioned rows: the per-row kernel (one evaluation of the map per
    row, for maps that keep rows contiguous and 16-byte vectors) and the per-vector kernel."""
    vt, tio, torch = gpu
    rng = np.random.default_rng(7)
    B, win = 3 if R == 9 else 2, 3
    x = workloads.encode((rng.normal(size=(B, R, R, C)) * 2 + 0.5).astype(np.float32), dtype)
    nw = R // win
    chain = [("x1", "reshape", ("X",), {"shape": (B, nw, win, nw, win, C)}),
             ("x2", "permute", ("x1",), {"perm": (0, 1, 3, 2, 4, 5)}),
             ("T0" if cut else "T", "reshape", ("x2",), {"shape": (B * nw * nw, win * win, C)})]
    if cut:
        chain.append(("T", "slice", ("T0",), {"dim": 2, "start": cut, "stop": C, "step": 1}))
    wl = workloads.Workload("ln", dtype, {"X": x}, chain, {"kind": "materialize", "x": "T"})
    dense = dm_ops.run_chain(chain, wl.sources)["T"]
    ref = consumers.layernorm(consumers.decode(dense, dtype), 1e-5)
    dw = tio.DeviceWorkload(wl)
    d = dw.build("T")
    out, check = guarded(torch, tio, dense.shape, dtype)
    vt.vt_elementwise(vt.EW_LAYERNORM, d, None, 1e-5, out)
    torch.cuda.synchronize()
    got = tio.to_host_f64(out)
    tol = {"f32": 2e-6, "f16": 2e-3, "bf16": 1.6e-2}[dtype]      # output rounding of values up to ~4
    assert np.max(np.abs(got - ref)) <= tol * max(1.0, np.max(np.abs(ref)))
    check()


# ------------------------------------------------------------------ block-wise paths
def guarded(torch, tio, shape, dtype, pad=4096):
    """A device buffer with canary bytes before and after the tensor: (tensor view, check)."""
    td = tio.TORCH_DTYPE[dtype]
    esz = torch.empty(0, dtype=td).element_size()
    n = int(np.prod(shape))
    raw = torch.full((2 * pad + n * esz,), 0xA5, dtype=torch.uint8, device="cuda:0")
    view = raw[pad:pad + n * esz].view(td).view(*shape)

    def check():
        host = raw.cpu().numpy()
        assert (host[:pad] == 0xA5).all() and (host[pad + n * esz:] == 0xA5).all(), "write outside the destination"

    return view, check


BLOCK_CASES = [
    # name, source shapes, chain, result: block sizes from 32 bytes to 1 KB, ragged block counts,
    # fewer blocks than a wave takes per round, pieces and tables
    ("heads_d16", {"X": (3, 5, 37, 16)}, [("p", "permute", ("X",), {"perm": (0, 2, 1, 3)}), ("R", "reshape", ("p",), {"shape": (111, 80)})]),
    ("heads_d32", {"X": (2, 7, 50, 32)}, [("p", "permute", ("X",), {"perm": (0, 2, 1, 3)}), ("R", "reshape", ("p",), {"shape": (100, 224)})]),
    ("heads_d128", {"X": (2, 6, 300, 128)}, [("p", "permute", ("X",), {"perm": (0, 2, 1, 3)}), ("R", "reshape", ("p",), {"shape": (600, 768)})]),
    ("heads_d512", {"X": (2, 3, 41, 512)}, [("p", "permute", ("X",), {"perm": (0, 2, 1, 3)}), ("R", "reshape", ("p",), {"shape": (82, 1536)})]),
    ("rows_2048", {"X": (97, 2048)}, [("R", "index_select", ("X",), {"dim": 0, "index": "t"})]),
    ("concat_cols", {"X": (33, 64), "Y": (33, 192)}, [("R", "concat", ("X", "Y"), {"dim": 1})]),
    ("concat_rows", {"X": (24, 40), "Y": (8, 40)}, [("R", "concat", ("X", "Y"), {"dim": 0})]),
    ("expand_heads", {"X": (2, 3, 70, 64)}, [("u", "unsqueeze", ("X",), {"dim": 2}), ("e", "expand", ("u",), {"shape": (2, 3, 4, 70, 64)}),
                                             ("R", "reshape", ("e",), {"shape": (2, 12, 70, 64)})]),
    ("window", {"X": (2, 14, 14, 64)}, [("a", "reshape", ("X",), {"shape": (2, 2, 7, 2, 7, 64)}), ("b", "permute", ("a",), {"perm": (0, 1, 3, 2, 4, 5)}),
                                        ("R", "reshape", ("b",), {"shape": (8, 49, 64)})]),
    ("tiny", {"X": (2, 3, 16)}, [("R", "permute", ("X",), {"perm": (1, 0, 2)})]),
    # pieces that do not span a middle dim, behind a permute: the term form tests that dim's
    # coordinate and takes its digits from the local coordinate
    ("concat_mid_permuted", {"X": (3, 20, 5, 32), "Y": (3, 13, 5, 32)},
     [("c", "concat", ("X", "Y"), {"dim": 1}), ("R", "permute", ("c",), {"perm": (2, 0, 1, 3)})]),
    ("three_pieces", {"X": (41, 32), "Y": (41, 96), "W": (41, 64)},
     [("c", "concat", ("X", "Y"), {"dim": 1}), ("R", "concat", ("c", "W"), {"dim": 1})]),
    ("sliced_heads_concat", {"X": (2, 4, 60, 64), "Y": (2, 4, 7, 64)},
     [("s", "slice", ("X",), {"dim": 2, "start": 3, "stop": 51, "step": 1}), ("c", "concat", ("s", "Y"), {"dim": 2}),
      ("p", "permute", ("c",), {"perm": (0, 2, 1, 3)}), ("R", "reshape", ("p",), {"shape": (110, 256)})]),
    ("split_reshaped", {"X": (6, 8, 96)},
     [("s", "split", ("X",), {"dim": 2, "sizes": (32, 64), "output": 1}), ("p", "permute", ("s",), {"perm": (1, 0, 2)}),
      ("R", "reshape", ("p",), {"shape": (8, 384)})]),
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("name,shapes,chain", BLOCK_CASES, ids=[c[0] for c in BLOCK_CASES])
def test_materialize_block_paths_bit_exact_with_canaries(gpu, name, shapes, chain, dtype):
    vt, tio, torch = gpu
    rng = np.random.default_rng(11)
    src = {k: workloads.encode(rng.normal(size=s).astype(np.float32), dtype) for k, s in shapes.items()}
    tables = {"t": rng.integers(0, 97, size=150).astype(np.int32)}
    wl = workloads.Workload(name, dtype, src, chain, {"kind": "materialize", "x": "R"}, tables)
    dense = dm_ops.run_chain(chain, wl.sources, tables)["R"]
    dw = tio.DeviceWorkload(wl)
    d = dw.build("R")
    assert d.block(512) * dense.dtype.itemsize >= 32, "case meant for the block path"
    # which of the two sources of block addresses the launch uses: the term form for every case
    # without an index table, the evaluator for the one with
    be = d.block(1024 // dense.dtype.itemsize)
    while dense.size % be:
        be //= 2
    assert (d.walk_addresses(be, 0, 0) is not None) == (name != "rows_2048"), name
    out, check = guarded(torch, tio, dense.shape, dtype)
    vt.vt_materialize(d, out)
    torch.cuda.synchronize()
    assert np.array_equal(bits(tio.to_host_bits(out)), bits(dense)), d.dump()
    check()


TRANSPOSE_CASES = [
    # source shape, perm: the source's contiguous dim is not the result's innermost one
    ((100, 130), (1, 0)),                      # plain 2-D transpose, ragged tiles
    ((64, 64), (1, 0)),                        # exactly one tile
    ((3, 70, 96), (0, 2, 1)),                  # batched
    ((5, 33, 7, 40), (3, 1, 2, 0)),            # the two directions far apart, two other digits
    ((2, 200, 3, 17), (0, 3, 2, 1)),           # 17 >= 16: still tiled
    ((6, 9, 50), (2, 0, 1)),                   # digits of the source's other dims merge (6 x 9 contiguous rows)
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape,perm", TRANSPOSE_CASES)
def test_materialize_transposes_bit_exact_with_canaries(gpu, shape, perm, dtype):
    """Permutes that move the source's contiguous dim away from the innermost place: the tiled
    transposing copy (and, for the chains that do not fit its form, the per-vector kernel)."""
    vt, tio, torch = gpu
    rng = np.random.default_rng(31)
    src = {"X": workloads.encode(rng.normal(size=shape).astype(np.float32), dtype)}
    chain = [("R", "permute", ("X",), {"perm": perm})]
    wl = workloads.Workload("transpose", dtype, src, chain, {"kind": "materialize", "x": "R"})
    dense = dm_ops.run_chain(chain, wl.sources)["R"]
    dw = tio.DeviceWorkload(wl)
    d = dw.build("R")
    assert d.block(512) * dense.dtype.itemsize < 32, "case meant for maps without blocks"
    out, check = guarded(torch, tio, dense.shape, dtype)
    vt.vt_materialize(d, out)
    torch.cuda.synchronize()
    assert np.array_equal(bits(tio.to_host_bits(out)), bits(dense)), d.dump()
    check()
    # the same through the one-operator copy of the materialized paths
    out2, check2 = guarded(torch, tio, dense.shape, dtype)
    vt.vt_copy_op("permute", [(shape, dtype, dw.tensors["X"].data_ptr())], {"perm": perm}, out2)
    torch.cuda.synchronize()
    assert np.array_equal(bits(tio.to_host_bits(out2)), bits(dense))
    check2()


def test_scatter_block_path_round_trip_with_canaries(gpu):
    """Store direction on the block path: a dense tensor written through the permuted map, every
    other byte of the target left alone, then read back through the same map."""
    vt, tio, torch = gpu
    rng = np.random.default_rng(12)
    chain = [("s", "slice", ("T",), {"dim": 2, "start": 5, "stop": 35, "step": 1}),       # [4,6,30,64] of [4,6,40,64]
             ("p", "permute", ("s",), {"perm": (0, 2, 1, 3)}), ("R", "reshape", ("p",), {"shape": (120, 384)})]
    target0 = workloads.encode(rng.normal(size=(4, 6, 40, 64)).astype(np.float32), "bf16")
    vals = workloads.encode(rng.normal(size=(120, 384)).astype(np.float32), "bf16")
    want = dm_ops.store_through(chain, {"T": target0}, "R", vals)["T"]
    tgt, check = guarded(torch, tio, target0.shape, "bf16")
    tgt.copy_(tio.to_device(target0, "bf16"))
    dv = tio.to_device(vals, "bf16")
    src = vt.build_chain([], {"V": (vals.shape, "bf16", dv.data_ptr())}, "V")
    dst = vt.build_chain(chain, {"T": (target0.shape, "bf16", tgt.data_ptr())}, "R")
    assert dst.block(512) == 64
    vt.vt_scatter(src, dst)
    torch.cuda.synchronize()
    assert np.array_equal(tio.to_host_bits(tgt), want)
    check()
    back, check2 = guarded(torch, tio, vals.shape, "bf16")
    vt.vt_materialize(dst, back)
    torch.cuda.synchronize()
    assert np.array_equal(tio.to_host_bits(back), vals)
    check2()


ROWSUM_CASES = [
    # rows, (A, B, C0) of X[A,B,C0] -> permute(1,0,2) -> reshape [B, A*C0], Y columns: blocks of C0 (X part),
    # of gcd with the Y part, several cursor reloads per row (more than 64 blocks), ragged last window
    (5, (3, 5, 16), 16),
    (9, (70, 9, 16), 48),          # 70 blocks of 16 + 3: the block cursor is reloaded inside a row
    (4, (2, 4, 1024), 512),        # blocks longer than a window of 64 columns
    (6, (5, 6, 80), 16),           # 80 = 16 * 5: blocks of 16
    (3, (40, 3, 128), 1024 + 64),  # the unrolled 512-column loop and its remainder
]


@pytest.mark.parametrize("rows,xs,ny", ROWSUM_CASES)
def test_add_rowsum_block_path_bit_exact(gpu, rows, xs, ny):
    vt, tio, torch = gpu
    rng = np.random.default_rng(13)
    A, B, C0 = xs
    assert B == rows
    C = A * C0 + ny
    src = {"X": rng.normal(size=xs).astype(np.float32), "Y": rng.normal(size=(B, ny)).astype(np.float32),
           "Z": rng.normal(size=(B, C)).astype(np.float32)}
    chain = [("p", "permute", ("X",), {"perm": (1, 0, 2)}), ("r", "reshape", ("p",), {"shape": (B, A * C0)}),
             ("V", "concat", ("r", "Y"), {"dim": 1})]
    wl = workloads.Workload("rowsum_blocks", "f32", src, chain, {"kind": "add_rowsum", "x": "V", "y": "Z"})
    ref = run_workload(wl)
    dw = tio.DeviceWorkload(wl)
    v, z = dw.build("V"), dw.build("Z")
    assert v.block() >= 16
    be = v.block()
    while C % be:
        be //= 2
    assert v.row_walk(be) and z.row_walk(z.block(C & -C)), "these maps resolve on the host: the kernel takes block addresses from segments"
    out, check = guarded(torch, tio, (B,), "f32")
    vt.vt_elementwise(vt.EW_ADD_ROWSUM, v, z, 0.0, out)
    torch.cuda.synchronize()
    assert np.array_equal(bits(out.cpu().numpy()), bits(ref["out"]))
    check()


@pytest.mark.parametrize("rows,cols,ny", [(37, 64, 16), (130, 1024, 256), (9, 4160, 64)])
def test_add_rowsum_block_path_through_the_evaluator_bit_exact(gpu, rows, cols, ny):
    """Rows gathered through an index table: the host cannot resolve the map into segments, and the
    block addresses come from the evaluator (one evaluation per block)."""
    vt, tio, torch = gpu
    rng = np.random.default_rng(17)
    C = cols + ny
    src = {"X": rng.normal(size=(rows + 5, cols)).astype(np.float32), "Y": rng.normal(size=(rows, ny)).astype(np.float32),
           "Z": rng.normal(size=(rows, C)).astype(np.float32)}
    idx = rng.integers(0, rows + 5, size=rows).astype(np.int32)
    chain = [("g", "index_select", ("X",), {"dim": 0, "index": "I"}), ("V", "concat", ("g", "Y"), {"dim": 1})]
    wl = workloads.Workload("rowsum_gathered", "f32", src, chain, {"kind": "add_rowsum", "x": "V", "y": "Z"}, {"I": idx})
    ref = run_workload(wl)
    dw = tio.DeviceWorkload(wl)
    v, z = dw.build("V"), dw.build("Z")
    assert v.block() >= 16 and v.row_walk(min(v.block(), C & -C)) == []
    out, check = guarded(torch, tio, (rows,), "f32")
    vt.vt_elementwise(vt.EW_ADD_ROWSUM, v, z, 0.0, out)
    torch.cuda.synchronize()
    assert np.array_equal(bits(out.cpu().numpy()), bits(ref["out"]))
    check()


def test_add_rowsum_random_chains_bit_exact(gpu):
    """Random chains seen as [R, C] for every split of their dims, added to a dense operand and
    summed by rows: bit for bit the oracle's fixed-order sum, whether the kernel takes its block
    addresses from host-resolved segments (one or two levels, several pieces, any block size) or
    from the evaluator."""
    vt, tio, torch = gpu
    rng = np.random.default_rng(23)
    walked = evaluated = 0
    for seed in range(100):
        wl = workloads.random_chain(seed, n_ops=4, max_extent=8)
        dense = dm_ops.run_chain(wl.chain, wl.sources, wl.index_tables)["R"]
        shape = dense.shape
        n = int(np.prod(shape))
        for cut in range(len(shape) + 1):
            rows = int(np.prod(shape[:cut]))
            cols = n // rows
            z = rng.normal(size=(rows, cols)).astype(np.float32) * 8.0
            src = dict(wl.sources)
            src["Zr"] = z
            chain = list(wl.chain) + [("R2", "reshape", ("R",), {"shape": (rows, cols)})]
            wl2 = workloads.Workload("rowsum_random", "f32", src, chain, {"kind": "add_rowsum", "x": "R2", "y": "Zr"}, wl.index_tables)
            dw = tio.DeviceWorkload(wl2)
            try:
                v, zd = dw.build("R2"), dw.build("Zr")
            except vt.VtError as e:
                assert e.code == vt.ERR_UNSUPPORTED
                continue
            be = v.block()
            while cols % be:
                be //= 2
            ref = consumers.add_rowsum_f32(np.ascontiguousarray(dense.reshape(rows, cols)), z)
            out, check = guarded(torch, tio, (rows,), "f32")
            try:
                vt.vt_elementwise(vt.EW_ADD_ROWSUM, v, zd, 0.0, out)
            except vt.VtError as e:
                assert e.code == vt.ERR_UNSUPPORTED, str(e)     # more pieces than the device form of a map holds
                continue
            torch.cuda.synchronize()
            if v.row_walk(be):
                walked += 1
            else:
                evaluated += 1
            assert np.array_equal(bits(out.cpu().numpy()), bits(ref)), (seed, cut, v.dump())
            check()
    assert walked >= 100 and evaluated >= 100, (walked, evaluated)


def test_add_rowsum_at_a_memory_bound_size_bit_exact(gpu):
    """The elementwise consumer at the size the benchmark times it (335 MB read), against the
    oracle's fixed-order sum, bit for bit, virtual and through the lean materialized path."""
    vt, tio, torch = gpu
    from paper_2604_09558_amd import pipelines
    wl = workloads.rowsum_chain_large()
    ref = run_workload(wl)["out"]
    dw = tio.DeviceWorkload(wl)
    p = pipelines.make_pipeline(dw)
    assert p.x.block() == 128
    p.run()
    torch.cuda.synchronize()
    assert np.array_equal(bits(p.out.cpu().numpy()), bits(ref))
    lean = pipelines.make_lean_pipeline(dw)
    lean.run()
    torch.cuda.synchronize()
    assert np.array_equal(bits(lean.consumer.out.cpu().numpy()), bits(ref))
