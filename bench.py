#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

One "step" runs every kernel of the path once on its full-size synthetic
configuration (inputs resident in HBM): SpMV on DIA/CSR (7-diagonal banded
matrix), ELL/CSR (bounded row lengths), unsorted / sorted COO and CSR
(power-law rows), the COO->CSR conversion, and TTV / MTTKRP on 3rd-order
COO / CSF. Prints ONE JSON line. The headline is the SpMV table: `per_format`
holds, for each of the four formats at its largest configuration, GFLOP/s,
algorithmic GB/s and its fraction of the 8 TB/s HBM peak (and, where the
columns are random, the fraction of the machine's measured gather rate);
`value` is their aggregate GFLOP/s; `roofline` is the format furthest below
the 60 % target. `kernels` lists every call of the step, `cpu_baseline` the
oracle's plain loops timed on the host.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only name,name] [--scale S]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Item:
    """One kernel call of the step with its algorithmic work."""

    def __init__(self, name, run, flops, bytes_, note="", gathers=0, gather_table=None):
        self.name, self.run, self.flops, self.bytes, self.note = name, run, flops, bytes_, note
        # random gathers the call performs and the ceiling entry they are compared with
        self.gathers, self.gather_table = gathers, gather_table
        self.events = []


def build_items(args):
    import torch
    import paper_1804_10112_amd as spt
    import workloads as wl

    dev = "cuda:0"
    items, cpu_jobs, keep = [], [], []
    s = args.scale

    def up(a):
        t = torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        keep.append(t)
        return t

    def spmv_item(name, spec, x_np, bytes_, flops, fmt, gather_table=None, note=""):
        A = spt.DeviceTensor(spec)
        x = up(x_np)
        y = torch.empty(spec.dims[0], dtype=A.torch_dtype, device=dev)
        ws = A.workspace(spt.SPT_OP_SPMV)
        keep.extend([A, y, ws])
        items.append(Item(name, lambda: spt.spt_spmv(A, x, y, ws), flops, bytes_, note,
                          gathers=flops // 2 if gather_table else 0, gather_table=gather_table))
        cpu_jobs.append((name, lambda o, nat, t=spec, v=x_np, f=fmt: o.plain_spmv(t, v, f, native=nat), flops,
                         fmt != "coo"))
        return A, x, y

    def unhinted(spec):
        """CSR as the paper has it: pos and crd only, no declared bound on the row length."""
        lv = spec.levels[1]
        return wl.csr_spec(spec.dims[0], spec.dims[1], lv.pos, lv.crd, spec.vals, name=spec.name)

    want = set(args.only.split(",")) if args.only else None

    def on(name):
        if want is None:
            return name not in ("x14", "x16", "n2", "n3", "n4", "n5", "n6")   # these groups run only on request
        return name in want or name.split("_")[0] in want

    # ---- config 2: banded, 7 diagonals, fp64: DIA and CSR
    def group_c2():
        t0 = time.time()
        c2 = wl.config2(N=max(64, int(2_000_000 * s)))
        N, nnz = c2["dia"].dims[0], c2["nnz"]
        K = c2["dia"].levels[0].N
        log(f"c2 generated in {time.time()-t0:.1f}s: N={N} nnz={nnz}")
        spmv_item("c2_dia_spmv", c2["dia"], c2["x"], 8 * nnz + 4 * K + 16 * N, 2 * nnz, "dia",
                  note="bytes: in-range cells only")
        spmv_item("c2_csr_spmv", unhinted(c2["csr"]), c2["x"], 12 * nnz + 4 * (N + 1) + 16 * N, 2 * nnz, "csr")
        del c2
    # ---- config 3: row lengths 8..32, fp32: ELL and CSR
    def group_c3():
        t0 = time.time()
        c3 = wl.config3(N=max(64, int(1_000_000 * s)))
        N, nnz, W = c3["ell"].dims[0], c3["nnz"], c3["W"]
        log(f"c3 generated in {time.time()-t0:.1f}s: N={N} nnz={nnz} W={W}")
        spmv_item("c3_ell_spmv", c3["ell"], c3["x"], 8 * W * N + 8 * N, 2 * nnz, "ell", "gather_f32_table_1M",
                  note="bytes: the whole W x N arrays (crd is read to find the padding)")
        spmv_item("c3_csr_spmv", unhinted(c3["csr"]), c3["x"], 8 * nnz + 4 * (N + 1) + 8 * N, 2 * nnz, "csr",
                  "gather_f32_table_1M")
        del c3
    # ---- config 4: power-law rows, fp64, unsorted COO: the three pipelines of Section 5.4
    def group_c4():
        t0 = time.time()
        n4 = max(1024, int(4_000_000 * s))
        c4 = wl.config4(N=n4, nnz_target=int(60_000_000 * s), max_row=max(8, int(200_000 * s)), with_sorted=True)
        N, nnz = n4, c4["nnz"]
        log(f"c4 generated in {time.time()-t0:.1f}s: N={N} nnz={nnz} longest row {c4['max_row_len']}")
        A, x, _ = spmv_item("c4_coo_unsorted_spmv", c4["coo"], c4["x"], 16 * nnz + 24 * N, 2 * nnz, "coo",
                            "gather_f64_table_4M")
        # COO -> CSR (sort by (row,col) + pos assembly); its outputs feed the next two items
        pos = torch.empty(N + 1, dtype=torch.int32, device=dev)
        crd = torch.empty(nnz, dtype=torch.int32, device=dev)
        vout = torch.empty(nnz, dtype=A.torch_dtype, device=dev)
        wsc = A.workspace(spt.SPT_OP_COO_TO_CSR)
        keep.extend([pos, crd, vout, wsc])
        passes = conversion_passes(N, N, nnz, spt.SPT_ORDER_ROW_COL)
        items.append(Item("c4_coo_to_csr", lambda: spt.spt_coo_to_csr(A, spt.SPT_ORDER_ROW_COL, pos, crd, vout, wsc),
                          0, conversion_bytes(passes, nnz, N),
                          f"{passes} passes over the (key, index) pairs + final gather + pos"))
        items[-1].run()
        torch.cuda.synchronize()
        rows_sorted = torch.repeat_interleave(torch.arange(N, dtype=torch.int32, device=dev),
                                              (pos[1:] - pos[:-1]).long())
        sorted_coo = wl.coo_spec(N, N, np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float64))
        As = spt.DeviceTensor(sorted_coo)      # descriptor shell; point it at the device arrays
        As.c.level[0].crd = rows_sorted.data_ptr()
        As.c.level[1].crd = crd.data_ptr()
        As.c.vals = vout.data_ptr()
        As.c.nvals = nnz
        csr_shell = wl.csr_spec(N, N, np.zeros(N + 1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float64))
        Ac = spt.DeviceTensor(csr_shell)
        Ac.c.level[1].pos = pos.data_ptr()
        Ac.c.level[1].crd = crd.data_ptr()
        Ac.c.vals = vout.data_ptr()
        Ac.c.nvals = nnz
        y2 = torch.empty(N, dtype=A.torch_dtype, device=dev)
        ws2 = torch.empty(spt.spt_workspace_bytes(spt.SPT_OP_SPMV, As), dtype=torch.uint8, device=dev)
        keep.extend([rows_sorted, As, Ac, y2, ws2])
        items.append(Item("c4_coo_sorted_spmv", lambda: spt.spt_spmv(As, x, y2, ws2), 2 * nnz, 16 * nnz + 16 * N,
                          gathers=nnz, gather_table="gather_f64_table_4M"))
        items.append(Item("c4_csr_spmv", lambda: spt.spt_spmv(Ac, x, y2, ws2), 2 * nnz,
                          12 * nnz + 4 * (N + 1) + 16 * N, "plain (pos, crd) descriptor, no declared row bound",
                          gathers=nnz, gather_table="gather_f64_table_4M"))
        # the same CSR with its longest row declared: the entry-balanced kernel
        Ab = spt.DeviceTensor(csr_shell)
        for src, dst in ((Ac.c, Ab.c),):
            dst.level[1].pos, dst.level[1].crd, dst.vals, dst.nvals = src.level[1].pos, src.level[1].crd, src.vals, src.nvals
        Ab.c.level[1].max_children = int(c4["max_row_len"])
        keep.append(Ab)
        items.append(Item("c4_csr_spmv_declared_long_rows", lambda: spt.spt_spmv(Ab, x, y2, ws2), 2 * nnz,
                          12 * nnz + 4 * (N + 1) + 16 * N, "max_children = longest row: entry-balanced kernel",
                          gathers=nnz, gather_table="gather_f64_table_4M"))
        # CPU leg: CSR SpMV on the same matrix (the generator's own sorted copy of the entries)
        hcsr = wl.csr_from_sorted_coo(N, N, *c4["sorted"])
        cpu_jobs.append(("c4_csr_spmv", lambda o_, nat, t=hcsr, v=c4["x"]: o_.plain_spmv(t, v, "csr", native=nat),
                         2 * nnz, True))
        del c4
    # ---- config 5: skewed 3rd-order tensor, fp32: TTV and MTTKRP on COO and CSF
    def group_c5():
        t0 = time.time()
        dims = tuple(max(16, int(d * s)) for d in (100_000, 80_000, 50_000))
        c5 = wl.config5(dims=dims, nnz=max(1000, int(50_000_000 * s)))
        nnz, J = c5["nnz"], c5["C"].shape[1]
        nfib = len(c5["csf"].levels[1].crd)
        log(f"c5 generated in {time.time()-t0:.1f}s: nnz={nnz} fibers={nfib}")
        Bc, Bf = spt.DeviceTensor(c5["coo"]), spt.DeviceTensor(c5["csf"])
        cv, Cm, Dm = up(c5["c"]), up(c5["C"]), up(c5["D"])
        oi = torch.empty(nnz, dtype=torch.int32, device=dev)
        oj = torch.empty(nnz, dtype=torch.int32, device=dev)
        ov = torch.empty(nnz, dtype=torch.float32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int64, device=dev)
        Aout = torch.empty(dims[0], J, dtype=torch.float32, device=dev)
        w_tc, w_tf = Bc.workspace(spt.SPT_OP_TTV), Bf.workspace(spt.SPT_OP_TTV)
        w_mc, w_mf = Bc.workspace(spt.SPT_OP_MTTKRP, J), Bf.workspace(spt.SPT_OP_MTTKRP, J)
        keep.extend([Bc, Bf, oi, oj, ov, cnt, Aout, w_tc, w_tf, w_mc, w_mf])
        dense = 4 * (dims[1] + dims[2] + dims[0]) * J
        items.append(Item("c5_ttv_coo", lambda: spt.spt_ttv(Bc, cv, oi, oj, ov, cnt, w_tc), 2 * nnz,
                          16 * nnz + 12 * nfib + 4 * dims[2]))
        items.append(Item("c5_ttv_csf", lambda: spt.spt_ttv(Bf, cv, None, None, ov, cnt, w_tf), 2 * nnz,
                          8 * nnz + 4 * (nfib + 1) + 4 * nfib + 4 * dims[2]))
        items.append(Item("c5_mttkrp_coo", lambda: spt.spt_mttkrp(Bc, Cm, Dm, J, Aout, w_mc), 3 * J * nnz,
                          16 * nnz + dense, "compulsory HBM bytes; factor rows are gathered from cache"))
        items.append(Item("c5_mttkrp_csf", lambda: spt.spt_mttkrp(Bf, Cm, Dm, J, Aout, w_mf),
                          2 * J * nnz + 2 * J * nfib, 8 * nnz + 8 * nfib + dense,
                          "compulsory HBM bytes; factor rows are gathered from cache"))
        cpu_jobs.append(("c5_ttv_coo", lambda o, nat, t=c5["coo"], c=c5["c"]: o.plain_ttv(t, c, "coo", native=nat),
                         2 * nnz, False))
        cpu_jobs.append(("c5_ttv_csf", lambda o, nat, t=c5["csf"], c=c5["c"]: o.plain_ttv(t, c, "csf", native=nat),
                         2 * nnz, True))
        cpu_jobs.append(("c5_mttkrp_coo", lambda o, nat, t=c5["coo"], C=c5["C"], D=c5["D"]:
                         o.plain_mttkrp(t, C, D, "coo", native=nat), 3 * J * nnz, False))
        cpu_jobs.append(("c5_mttkrp_csf", lambda o, nat, t=c5["csf"], C=c5["C"], D=c5["D"]:
                         o.plain_mttkrp(t, C, D, "csf", native=nat), 2 * J * nnz + 2 * J * nfib, True))
        del c5
    # ---- on request (--only x14): the other conversion order of Figure 14's pipeline: rows sorted,
    #      input order kept inside a row (enough for SpMV), on config 4's unsorted COO
    def group_x14():
        n4 = max(1024, int(4_000_000 * s))
        c4 = wl.config4(N=n4, nnz_target=int(60_000_000 * s), max_row=max(8, int(200_000 * s)))
        nnz = c4["nnz"]
        A = spt.DeviceTensor(c4["coo"])
        pos = torch.empty(n4 + 1, dtype=torch.int32, device=dev)
        crd = torch.empty(nnz, dtype=torch.int32, device=dev)
        vout = torch.empty(nnz, dtype=A.torch_dtype, device=dev)
        wsc = A.workspace(spt.SPT_OP_COO_TO_CSR)
        keep.extend([A, pos, crd, vout, wsc])
        for tag, order in (("row_stable", spt.SPT_ORDER_ROW_STABLE), ("row_col", spt.SPT_ORDER_ROW_COL)):
            passes = conversion_passes(n4, n4, nnz, order)
            items.append(Item(f"x14_coo_to_csr_{tag}",
                              lambda order=order: spt.spt_coo_to_csr(A, order, pos, crd, vout, wsc), 0,
                              conversion_bytes(passes, nnz, n4), f"{passes} passes"))
        del c4
    # ---- on request (--only x16): CSR SpMV on config 3's matrix with x as dense array,
    #      sparse vector and hash map at three densities (the experiment of Figure 16)
    def group_x16():
        c3 = wl.config3(N=max(64, int(1_000_000 * s)))
        N, nnz = c3["csr"].dims[0], c3["nnz"]
        A = spt.DeviceTensor(c3["csr"])
        y = torch.empty(N, dtype=torch.float32, device=dev)
        ws = A.workspace(spt.SPT_OP_SPMV_SPARSE_X)
        keep.extend([A, y, ws])
        for dens in (1e-4, 1e-2, 0.5):
            nx = max(1, int(N * dens))
            xc, xv = wl.random_sparse_vector(N, nx, seed=7, dtype=np.float32, dist="n01")
            xd = np.zeros(N, np.float32)
            xd[xc] = xv
            xdense = up(xd)
            W = 1 << int(np.ceil(np.log2(2 * nx + 1)))      # load factor <= 0.5
            Xs = spt.DeviceTensor(wl.sparse_vector_spec(N, xc, xv))
            Xh = spt.DeviceTensor(wl.hash_vector_spec(N, xc, xv, W))
            keep.extend([Xs, Xh])
            tag = f"x16_d{dens:g}"
            items.append(Item(tag + "_dense", lambda xdense=xdense: spt.spt_spmv(A, xdense, y, ws),
                              2 * nnz, 8 * nnz + 12 * N))
            items.append(Item(tag + "_sparse", lambda Xs=Xs: spt.spt_spmv_sparse_x(A, Xs, y, ws),
                              2 * nnz, 8 * nnz + 8 * N + 8 * nx))
            items.append(Item(tag + "_hash", lambda Xh=Xh: spt.spt_spmv_sparse_x(A, Xh, y, ws),
                              2 * nnz, 8 * nnz + 8 * N + 8 * W))
        del c3
    # ---- on request (--only n2): INNERPROD (Section 5.3) on config 5's tensor, with itself
    #      and with a tensor holding every third of its coordinates
    def group_n2():
        dims = tuple(max(16, int(d * s)) for d in (100_000, 80_000, 50_000))
        c5 = wl.config5(dims=dims, nnz=max(1000, int(50_000_000 * s)))
        b = c5["coo"]
        nnz = c5["nnz"]
        i, j, k = (np.asarray(L.crd) for L in b.levels)
        sel = np.arange(0, nnz, 3)
        third = wl.coo3_spec(dims, i[sel], j[sel], k[sel], b.vals[sel])
        Bc, Bt = spt.DeviceTensor(b), spt.DeviceTensor(third)
        alpha = torch.zeros(1, dtype=torch.float32, device=dev)
        w1, w2 = Bc.workspace(spt.SPT_OP_INNERPROD), Bt.workspace(spt.SPT_OP_INNERPROD)
        keep.extend([Bc, Bt, alpha, w1, w2])
        items.append(Item("n2_innerprod_self", lambda: spt.spt_innerprod(Bc, Bc, alpha, w1),
                          2 * nnz, 32 * nnz))
        items.append(Item("n2_innerprod_third", lambda: spt.spt_innerprod(Bc, Bt, alpha, w1),
                          2 * len(sel), 16 * nnz + 16 * len(sel)))
        items.append(Item("n2_innerprod_third_rev", lambda: spt.spt_innerprod(Bt, Bc, alpha, w2),
                          2 * len(sel), 16 * nnz + 16 * len(sel)))
        # TTM (Section 5.3) with K = 32 on the same tensor, COO and CSF
        K = 32
        Bf = spt.DeviceTensor(c5["csf"])
        nfib = len(c5["csf"].levels[1].crd)
        Ck = up(np.random.default_rng(9).uniform(0, 1, (K, dims[2])).astype(np.float32))
        ti = torch.empty(nnz, dtype=torch.int32, device=dev)
        tj = torch.empty(nnz, dtype=torch.int32, device=dev)
        tv = torch.empty(nfib, K, dtype=torch.float32, device=dev)
        tcnt = torch.zeros(1, dtype=torch.int64, device=dev)
        w3, w4 = Bc.workspace(spt.SPT_OP_TTM, K), Bf.workspace(spt.SPT_OP_TTM, K)
        keep.extend([Bf, ti, tj, tv, tcnt, w3, w4])
        out_b = 4 * K * nfib
        items.append(Item("n2_ttm_coo", lambda: spt.spt_ttm(Bc, Ck, K, ti, tj, tv, tcnt, w3),
                          2 * K * nnz, 16 * nnz + 8 * nfib + out_b, "output fibres dominate the bytes"))
        items.append(Item("n2_ttm_csf", lambda: spt.spt_ttm(Bf, Ck, K, None, None, tv, tcnt, w4),
                          2 * K * nnz, 8 * nnz + 4 * nfib + out_b, "output fibres dominate the bytes"))
        # SpDM (Figure 11) with 32 columns: config 3's matrix as ordered COO (fp32) times a dense matrix
        c3 = wl.config3(N=max(64, int(1_000_000 * s)))
        N3, nnz3 = c3["csr"].dims[0], c3["nnz"]
        (r3, q3), v3 = oracle_free_coo(c3["csr"])
        Am = spt.DeviceTensor(wl.coo_spec(N3, N3, r3, q3, v3))
        Cd = up(np.random.default_rng(10).uniform(0, 1, (N3, 32)).astype(np.float32))
        Ad = torch.empty(N3, 32, dtype=torch.float32, device=dev)
        w5 = Am.workspace(spt.SPT_OP_SPDM, 32)
        keep.extend([Am, Ad, w5])
        items.append(Item("n2_spdm_coo", lambda: spt.spt_spdm(Am, Cd, 32, Ad, w5), 2 * 32 * nnz3,
                          12 * nnz3 + 2 * 4 * 32 * N3, "compulsory HBM bytes; rows of C are gathered from cache"))
        del c5
    # ---- on request (--only n3): sparse addition with sparse result. PLUS on config 5's tensor
    #      and a 10M-entry tensor of the same generator; COO and CSR matrix addition on config 4's
    #      sorted matrix and every second of its entries
    def group_n3():
        dims = tuple(max(16, int(d * s)) for d in (100_000, 80_000, 50_000))
        c5 = wl.config5(dims=dims, nnz=max(1000, int(50_000_000 * s)))
        nb = c5["nnz"]
        ci, cj, ck, cv = wl.random_coo3_entries(dims, max(200, int(10_000_000 * s)), wl.SEED_BASE + 55,
                                                np.float32, "u01", skew=1.5)
        Bc, Cc = spt.DeviceTensor(c5["coo"]), spt.DeviceTensor(wl.coo3_spec(dims, ci, cj, ck, cv))
        nc = len(cv)
        cap = nb + nc
        o0, o1, o2 = (torch.empty(cap, dtype=torch.int32, device=dev) for _ in range(3))
        ov = torch.empty(cap, dtype=torch.float32, device=dev)
        ocnt = torch.zeros(1, dtype=torch.int64, device=dev)
        wsa = torch.empty(spt.spt_add_workspace_bytes(Bc, Cc), dtype=torch.uint8, device=dev)
        keep.extend([Bc, Cc, o0, o1, o2, ov, ocnt, wsa])
        items.append(Item("n3_plus_coo3", lambda: spt.spt_add(Bc, Cc, None, o0, o1, o2, ov, ocnt, wsa),
                          nc, 32 * (nb + nc), "read 16 B + write <= 16 B per stored entry"))
        del c5
        n4 = max(1024, int(4_000_000 * s))
        c4 = wl.config4(N=n4, nnz_target=int(60_000_000 * s), max_row=max(8, int(200_000 * s)), with_sorted=True)
        rs, cs, vs = c4["sorted"]
        half = slice(0, len(vs), 2)
        nb, nc = len(vs), len(vs[half])
        cap = nb + nc
        q0, q1 = (torch.empty(cap, dtype=torch.int32, device=dev) for _ in range(2))
        qpos = torch.empty(n4 + 1, dtype=torch.int32, device=dev)
        qv = torch.empty(cap, dtype=torch.float64, device=dev)
        for fmt, mk in (("coo", wl.coo_spec), ("csr", wl.csr_from_sorted_coo)):
            Bm = spt.DeviceTensor(mk(n4, n4, rs, cs, vs))
            Cm2 = spt.DeviceTensor(mk(n4, n4, rs[half], cs[half], 0.5 * vs[half]))
            wsm = torch.empty(spt.spt_add_workspace_bytes(Bm, Cm2), dtype=torch.uint8, device=dev)
            keep.extend([Bm, Cm2, wsm])
            if fmt == "coo":
                run = lambda Bm=Bm, Cm2=Cm2, wsm=wsm: spt.spt_add(Bm, Cm2, None, q0, q1, None, qv, ocnt, wsm)
                byt = 16 * (nb + nc) + 16 * nb
            else:
                run = lambda Bm=Bm, Cm2=Cm2, wsm=wsm: spt.spt_add(Bm, Cm2, qpos, None, q1, None, qv, ocnt, wsm)
                byt = 12 * (nb + nc) + 12 * nb + 12 * (n4 + 1)
            items.append(Item(f"n3_add_{fmt}", run, nc, byt))
        # the running example: a CSR matrix times a COO matrix, element by element (result CSR)
        Cm3 = spt.DeviceTensor(wl.coo_spec(n4, n4, rs[half], cs[half], 0.5 * vs[half]))
        wsx = torch.empty(spt.spt_add_workspace_bytes(Bm, Cm3), dtype=torch.uint8, device=dev)
        keep.extend([Cm3, wsx])
        items.append(Item("n3_mul_csr_coo", lambda: spt.spt_mul(Bm, Cm3, qpos, None, q1, None, qv, ocnt, wsx),
                          nc, 12 * nb + 16 * nc + 12 * nc + 8 * (n4 + 1),
                          "read B (pos, cols, values) and C (16 B), write the common entries (12 B) and pos"))
        keep.extend([q0, q1, qpos, qv])
        del c4
    # ---- on request (--only n4): packers. Config 5's COO -> CSF, config 3's CSR -> ELL,
    #      config 2's matrix (as COO) -> DIA offsets + values
    def group_n4():
        dims = tuple(max(16, int(d * s)) for d in (100_000, 80_000, 50_000))
        c5 = wl.config5(dims=dims, nnz=max(1000, int(50_000_000 * s)))
        nnz = c5["nnz"]
        nfib, nsl = len(c5["csf"].levels[1].crd), len(c5["csf"].levels[0].crd)
        Bc = spt.DeviceTensor(c5["coo"])
        i32 = lambda m: torch.empty(m, dtype=torch.int32, device=dev)
        pk = [i32(2), i32(nnz), i32(nnz + 1), i32(nnz), i32(nnz + 1), i32(nnz)]
        pv = torch.empty(nnz, dtype=torch.float32, device=dev)
        pc = torch.zeros(2, dtype=torch.int64, device=dev)
        wp = Bc.workspace(spt.SPT_OP_TO_CSF)
        keep.extend([Bc, pk, pv, pc, wp])
        items.append(Item("n4_coo3_to_csf", lambda: spt.spt_coo3_to_csf(Bc, *pk, pv, pc, wp), 0,
                          16 * nnz + 8 * nnz + 8 * nnz + 8 * nfib + 8 * nsl,
                          "(i,j) read twice (count, fill), k and values copied"))
        del c5
        c3 = wl.config3(N=max(64, int(1_000_000 * s)))
        N3, W3, nnz3 = c3["csr"].dims[0], c3["W"], c3["nnz"]
        Ac = spt.DeviceTensor(c3["csr"])
        ec = i32(W3 * N3)
        ev = torch.empty(W3 * N3, dtype=torch.float32, device=dev)
        el = torch.zeros(1, dtype=torch.int32, device=dev)
        keep.extend([Ac, ec, ev, el])
        items.append(Item("n4_csr_to_ell", lambda: spt.spt_to_ell(Ac, W3, ec, ev, el, None), 0,
                          8 * nnz3 + 4 * (N3 + 1) + 8 * W3 * N3))
        del c3
        c2 = wl.config2(N=max(64, int(2_000_000 * s)))
        cc, cv = oracle_free_coo(c2["csr"])
        N2 = c2["csr"].dims[0]
        Ad = spt.DeviceTensor(wl.coo_spec(N2, N2, cc[0], cc[1], cv))
        offs = i32(64)
        Kd = torch.zeros(1, dtype=torch.int64, device=dev)
        dv = torch.empty(7 * N2, dtype=torch.float64, device=dev)
        wd = Ad.workspace(spt.SPT_OP_DIA_OFFSETS)
        keep.extend([Ad, offs, Kd, dv, wd])
        items.append(Item("n4_coo_dia_offsets", lambda: spt.spt_coo_dia_offsets(Ad, offs, 64, Kd, wd), 0,
                          8 * len(cv) + 16 * 2 * N2))
        items[-1].run()
        torch.cuda.synchronize()
        items.append(Item("n4_coo_to_dia", lambda: spt.spt_coo_to_dia(Ad, 7, offs, dv), 0,
                          16 * len(cv) + 2 * 8 * 7 * N2, "zero fill + scattered values"))
        del c2
    # ---- on request (--only n5): compositions without a kernel of their own, read through the
    #      level functions per stored value: config 3's matrix as CSC and as DCSR (SpMV), and its
    #      ELL layout unpacked to COO
    def group_n5():
        c3 = wl.config3(N=max(64, int(1_000_000 * s)))
        N3, nnz3 = c3["csr"].dims[0], c3["nnz"]
        (rr, cc), vv = oracle_free_coo(c3["csr"])
        xg = up(c3["x"])
        yg = torch.empty(N3, dtype=torch.float32, device=dev)
        for nm, spec in (("csc", wl.csc_from_coo(N3, N3, rr, cc, vv)),
                         ("dcsr", wl.dcsr_from_sorted_coo(N3, N3, rr, cc, vv))):
            Ag = spt.DeviceTensor(spec)
            wg5 = Ag.workspace(spt.SPT_OP_SPMV)
            keep.extend([Ag, wg5])
            items.append(Item(f"n5_spmv_{nm}", lambda Ag=Ag, wg5=wg5: spt.spt_spmv(Ag, xg, yg, wg5), 2 * nnz3,
                              8 * nnz3 + 12 * N3,
                              "one atomic per stored value" if nm == "csc" else "CSR kernel over the stored rows"))
        # array-of-structs COO of the same matrix (entries in row order): pairs split, then COO kernels
        Aa = spt.DeviceTensor(wl.coo_aos_spec((N3, N3), (rr, cc), vv))
        wa = Aa.workspace(spt.SPT_OP_SPMV)
        keep.extend([Aa, wa])
        items.append(Item("n5_spmv_coo_aos", lambda: spt.spt_spmv(Aa, xg, yg, wa), 2 * nnz3,
                          12 * nnz3 + 16 * nnz3 + 8 * N3, "pairs split into the workspace (8 B read + 8 B written per entry), then sorted-COO SpMV"))
        Ae = spt.DeviceTensor(c3["ell"])
        cells = len(c3["ell"].vals)
        g0, g1 = (torch.empty(cells, dtype=torch.int32, device=dev) for _ in range(2))
        gv = torch.empty(cells, dtype=torch.float32, device=dev)
        gcnt = torch.zeros(1, dtype=torch.int64, device=dev)
        wg = Ae.workspace(spt.SPT_OP_TO_COO)
        keep.extend([Ae, g0, g1, gv, gcnt, wg, yg])
        items.append(Item("n5_ell_to_coo", lambda: spt.spt_to_coo(Ae, g0, g1, None, gv, gcnt, wg), 0,
                          2 * 8 * cells + 12 * nnz3, "cells read twice (count, fill)"))
        del c3
    # ---- on request (--only n6): a 4x4-blocked fp64 matrix (FEM-like band, 8..24 blocks per
    #      block row) as BCSR and as its CSR twin
    def group_n6():
        nbr = max(64, int(500_000 * s))
        w = wl.random_bcsr(nbr, nbr, 4, 4, 8, 24, seed=wl.SEED_BASE + 77, dtype=np.float64,
                           band=max(32, int(5000 * s)), with_csr=True)
        nblk = w["nblocks"]
        xb = up(w["x"])
        yb = torch.empty(nbr * 4, dtype=torch.float64, device=dev)
        for nm, spec, byt in (("bcsr", w["bcsr"], (128 + 4) * nblk + 4 * (nbr + 1) + 16 * 4 * nbr),
                              ("csr_twin", w["csr"], 12 * 16 * nblk + 4 * (4 * nbr + 1) + 16 * 4 * nbr)):
            Ab = spt.DeviceTensor(spec)
            wb = Ab.workspace(spt.SPT_OP_SPMV)
            keep.extend([Ab, wb])
            items.append(Item(f"n6_spmv_{nm}", lambda Ab=Ab, wb=wb: spt.spt_spmv(Ab, xb, yb, wb),
                              2 * 16 * nblk, byt))
        keep.append(yb)
        del w
    if on("c3"):
        group_c3()
    if on("c2"):
        group_c2()
    if on("c4"):
        group_c4()
    if on("c5"):
        group_c5()
    if on("x14"):
        group_x14()
    if on("x16"):
        group_x16()
    if on("n2"):
        group_n2()
    if on("n3"):
        group_n3()
    if on("n4"):
        group_n4()
    if on("n6"):
        group_n6()
    if on("n5"):
        group_n5()
    return items, cpu_jobs, keep


def conversion_passes(N, M, nnz, order):
    """Global passes over the records that spt_coo_to_csr makes for this input (mirrors the
    library's plan: 8-bit digits over the significant bits of the column, then of the row)."""
    bits = lambda d: max(1, int(np.ceil(np.log2(max(d, 2)))))
    rows = (bits(N) + 7) // 8
    return rows + ((bits(M) + 7) // 8 if order == 0 else 0)


def conversion_bytes(passes, nnz, N):
    """Algorithmic bytes of COO -> CSR with a P-pass sort: every pass reads and writes a 64-bit
    key and a 32-bit payload per entry (2 * 12 bytes), the final gather reads and writes column
    and value once more (2 * 12), the pos assembly reads the sorted rows (4) and writes pos."""
    return passes * 2 * 12 * nnz + 2 * 12 * nnz + 4 * nnz + 4 * (N + 1)


def oracle_free_coo(csr_spec):
    """(rows, cols), values of a CSR spec, expanded with numpy (input preparation only)."""
    pos = np.asarray(csr_spec.levels[1].pos)
    rows = np.repeat(np.arange(len(pos) - 1, dtype=np.int32), np.diff(pos))
    return (rows, np.asarray(csr_spec.levels[1].crd)), csr_spec.vals


def measure_ceilings():
    """Achievable ceilings of this machine for the two access patterns that bound the path:
    a pure streaming read (16 / 8 / 4 bytes per lane) and random gathers from tables of the
    sizes of config 3's x (1M fp32) and config 4's x (4M fp64) with the library's probe kernels,
    and the runtime's device-to-device copy."""
    import torch
    import paper_1804_10112_amd as spt
    dev = "cuda:0"
    out = {}
    nbytes = 1 << 30
    src = torch.zeros(nbytes // 4, dtype=torch.float32, device=dev)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)

    def timed(fn, reps=10):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps * 1e-3

    for lane in (16, 8, 4):
        t = timed(lambda: spt.spt_probe_read(src, nbytes, lane, sink))
        out[f"read_{lane}B_per_lane_GBs"] = round(nbytes / t / 1e9, 1)
    n = 1 << 25
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    for name, rows, tdt, sdt in (("gather_f32_table_1M", 1_000_000, torch.float32, spt.SPT_F32),
                                 ("gather_f64_table_4M", 4_000_000, torch.float64, spt.SPT_F64)):
        idx = torch.randint(0, rows, (n,), dtype=torch.int32, device=dev, generator=g)
        table = torch.zeros(rows, dtype=tdt, device=dev)
        o = torch.empty(n, dtype=tdt, device=dev)
        t = timed(lambda: spt.spt_probe_gather(idx, n, table, sdt, o))
        out[name + "_Gelem_s"] = round(n / t / 1e9, 1)
    # the runtime's own device-to-device copy: the yardstick for a radix pass (read + write)
    dst = torch.empty_like(src)
    t = timed(lambda: dst.copy_(src))
    out["copy_read_plus_write_GBs"] = round(2 * nbytes / t / 1e9, 1)
    del src, dst
    return out


def csrc_hash():
    """Hash of the kernel sources: measured traffic is only valid for the tree it was measured on."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_1804_10112_amd", "csrc", "*"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def read_traffic_file():
    """Bytes moved between the L2 caches and the fabric (Infinity Cache / HBM) per call, measured
    offline with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE) and kept as `name = bytes` lines in
    profiles/hbm_traffic_pmc.txt together with `csrc_hash = ...` of the tree they were measured
    on. Returns {} when the file is absent or belongs to other kernel sources."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_pmc.txt")
    out, tree = {}, None
    if os.path.exists(path):
        for line in open(path):
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = (t.strip() for t in line.split("="))
                if k == "csrc_hash":
                    tree = v
                else:
                    out[k] = int(float(v))
    if tree != csrc_hash():
        log(f"profiles/hbm_traffic_pmc.txt was measured on csrc {tree}, this tree is {csrc_hash()}: traffic = null")
        return {}
    return out


def config1_warm(reps=200):
    """Config 1 (4096 x 4096, 40 960 entries, fp64) fits every cache: its SpMV is bound by launch
    and dependent-load latency, not bandwidth. Warm back-to-back calls, microseconds per call."""
    import torch
    import paper_1804_10112_amd as spt
    import workloads as wl
    c1 = wl.config1()
    x = torch.from_numpy(c1["x"]).cuda()
    out = {}
    for fmt in ("csr", "coo"):
        A = spt.DeviceTensor(c1[fmt])
        y = torch.empty(c1[fmt].dims[0], dtype=torch.float64, device="cuda")
        ws = A.workspace(spt.SPT_OP_SPMV)
        # a tight caller resolves device pointers and the stream once, not per call
        stream = torch.cuda.current_stream().cuda_stream
        xp, yp = x.data_ptr(), y.data_ptr()
        for _ in range(10):
            spt.spt_spmv(A, xp, yp, ws, stream)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            spt.spt_spmv(A, xp, yp, ws, stream)
        b.record()
        torch.cuda.synchronize()
        out[f"{fmt}_spmv_us"] = round(a.elapsed_time(b) * 1e3 / reps, 2)
    return out


HEADLINE = {"dia": "c2_dia_spmv", "ell": "c3_ell_spmv", "csr": "c4_csr_spmv", "coo": "c4_coo_sorted_spmv"}
# the CPU's COO loop is the paper's order-independent scatter: it runs on the unsorted entries
CPU_HEADLINE = {"dia": "c2_dia_spmv", "ell": "c3_ell_spmv", "csr": "c4_csr_spmv", "coo": "c4_coo_unsorted_spmv"}


def cpu_baseline(cpu_jobs, target_s=8.0, max_rounds=12):
    """The oracle's plain per-format loops on the same full-size inputs, built for this host
    (gcc -O3 -march=native -fopenmp), in two legs: one thread (the paper's protocol) and all the
    cores this process may use (the loops over rows / fibres / slices run in parallel, the
    scatter loops of the COO kernels stay serial). Each leg: rounds of one call per job until
    about target_s seconds. `value` is the aggregate SpMV GFLOP/s over the four formats at their
    largest configuration, like the GPU headline."""
    import oracle
    ncores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    want = int(os.environ.get("OMP_NUM_THREADS", "0") or 0)
    ncores = min(ncores, want) if want > 0 else ncores

    def leg(threads):
        used = oracle.set_threads(threads)
        total_t, rounds, per_job = 0.0, 0, {}
        while rounds < max_rounds and total_t < target_s and cpu_jobs:
            for name, job, flops, parallel in cpu_jobs:
                t0 = time.perf_counter()
                job(oracle, True)
                dt = time.perf_counter() - t0
                total_t += dt
                per_job[name] = per_job.get(name, 0.0) + dt
            rounds += 1
        if total_t == 0:
            return None
        flops_of = {name: flops for name, _, flops, _ in cpu_jobs}
        head = [n for n in CPU_HEADLINE.values() if n in per_job]
        hf = sum(flops_of[n] for n in head)
        ht = sum(per_job[n] for n in head) / rounds
        detail = " ".join(f"{n}:{t / rounds * 1e3:.1f}ms" for n, t in per_job.items())
        serial = ", ".join(n for n, _, _, par in cpu_jobs if not par)
        return {"value": round(hf / ht / 1e9, 3) if ht > 0 else None, "unit": "GFLOP/s", "cores": used, "kind": "oracle",
                "sample": f"{rounds} rounds ({total_t:.1f} s) of one call per job of the oracle's plain loops on the "
                          f"full-size inputs, built {oracle.lib_native.flags}; value = flops / time summed over "
                          f"{', '.join(head)}; mean per call: {detail}"
                          + (f"; serial by construction (scatter loops): {serial}" if used > 1 and serial else "")}

    single = leg(1)
    allc = leg(ncores) if ncores > 1 else None
    if allc is None:
        return single
    allc["single_thread"] = single
    return allc


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--only", type=str, default="")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink every configuration (testing)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true")
    ap.add_argument("--flush-mb", type=int, default=0,
                    help="write a buffer of this many MiB before every call (outside its timed interval): "
                         "cold caches for partial runs with --only")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB streaming read and one 1 GiB fill per step (known traffic, "
                         "for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE); excluded from every figure")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported")

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    import paper_1804_10112_amd as spt

    items, cpu_jobs, keep = build_items(args)
    stream = torch.cuda.current_stream()
    calib = None
    if args.calib_copy:
        # known traffic: a 1 GiB streaming read (library probe) and a 1 GiB fill
        ca = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")
        sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")

        def calib():
            spt.spt_probe_read(ca, 1 << 30, 16, sink)
            ca.zero_()

    flush = None
    if args.flush_mb > 0:
        # a partial step (--only) leaves its few operands in the 256 MB Infinity Cache; writing a
        # large buffer before every call restores what the full step does by itself
        # (read, not written: in the full step a call follows kernels that mostly read, and
        # dirty lines left in the memory-side cache would charge their write-back to the call)
        flush = torch.zeros(args.flush_mb << 20, dtype=torch.uint8, device="cuda:0")
        flush_sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")

    def step(record):
        # one event between consecutive calls: the end of call k is the start of call k+1
        prev = None
        if record:
            prev = torch.cuda.Event(enable_timing=True)
            prev.record(stream)
        for it in items:
            if flush is not None:
                spt.spt_probe_read(flush, args.flush_mb << 20, 16, flush_sink)
                if record:
                    prev = torch.cuda.Event(enable_timing=True)
                    prev.record(stream)
            it.run()
            if record:
                e = torch.cuda.Event(enable_timing=True)
                e.record(stream)
                it.events.append((prev, e))
                prev = e
        if calib is not None:
            calib()

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    traffic = read_traffic_file()
    ceilings = None if args.no_ceilings else measure_ceilings()
    kernels = []
    for it in items:
        times = [a.elapsed_time(b) for a, b in it.events]
        ms = float(np.mean(times))
        gbs = it.bytes / (ms * 1e-3) / 1e9
        tr = traffic.get(it.name)
        k = {"name": it.name, "ms": round(ms, 4), "ms_median": round(float(np.median(times)), 4),
             "ms_min": round(float(np.min(times)), 4),
             "gflops": round(it.flops / (ms * 1e-3) / 1e9, 2),
             "alg_gbs": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
             "alg_bytes": it.bytes,
             # bytes between the L2 caches and the fabric (rocprofv3 counters, profiles/): lines
             # served by the Infinity Cache count too, so this is an upper bound on HBM traffic
             "l2_fabric_bytes": tr,
             "l2_fabric_over_algorithmic": round(tr / it.bytes, 2) if tr else None}
        if it.gathers:
            k["gathers"] = it.gathers
            k["gather_Gelem_s"] = round(it.gathers / (ms * 1e-3) / 1e9, 1)
            if ceilings and it.gather_table + "_Gelem_s" in ceilings:
                # second bound of a random-column kernel: its gathers per second over what the
                # probe (4 independent gathers per lane, same table size) reaches in this run
                k["gather_frac"] = round(k["gather_Gelem_s"] / ceilings[it.gather_table + "_Gelem_s"], 3)
        if it.note:
            k["note"] = it.note
        kernels.append(k)
    by_name = {k["name"]: k for k in kernels}
    per_format = {}
    for fmt, name in HEADLINE.items():
        if name in by_name:
            k = by_name[name]
            per_format[fmt] = {key: k.get(key) for key in ("name", "ms", "gflops", "alg_gbs", "frac_hbm_peak",
                                                           "gather_frac", "l2_fabric_over_algorithmic")}
            per_format[fmt]["meets_60pct"] = k["frac_hbm_peak"] >= 0.60
    head = [by_name[n] for n in HEADLINE.values() if n in by_name]
    if head:
        it_of = {it.name: it for it in items}
        value = sum(it_of[k["name"]].flops for k in head) / sum(k["ms"] * 1e-3 for k in head) / 1e9
        worst = min(head, key=lambda k: k["frac_hbm_peak"])
    else:   # a partial run without any of the four headline calls
        value = sum(it.flops for it in items) / (ms_per_step * 1e-3) / 1e9
        worst = max(kernels, key=lambda k: k["ms"])
    dom = max(kernels, key=lambda k: k["ms"])
    out = {
        "metric": "SpMV GFLOP/s + achieved HBM GB/s (% of peak) per format, 1 MI355X",
        "value": round(value, 2),
        "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64+f32", "data": "synthetic",
        "config": {"workload": "one pass over every kernel of the path at full size: "
                               + ", ".join(it.name for it in items)
                               + "; value = SpMV flops / SpMV time summed over the four formats at their largest "
                                 "configuration (" + ", ".join(f"{f}: {n}" for f, n in HEADLINE.items()) + ")",
                   "scale": args.scale},
        # the SpMV format furthest below the 60 % target; achieved = algorithmic bytes / event time
        "roofline": {"bound": "hbm", "kernel": worst["name"], "achieved": worst["alg_gbs"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": worst["frac_hbm_peak"],
                     "traffic": worst["l2_fabric_bytes"], "gather_frac": worst.get("gather_frac")},
        "per_format": per_format,
        "longest_call": {"name": dom["name"], "ms": dom["ms"], "frac_hbm_peak": dom["frac_hbm_peak"]},
        "step_gflops": round(sum(it.flops for it in items) / (ms_per_step * 1e-3) / 1e9, 2),
        "kernels": kernels,
        "library": spt.spt_version(),
        "csrc_hash": csrc_hash(),
    }
    if ceilings:
        out["ceilings"] = ceilings
        out["c1_warm"] = config1_warm()
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cpu_jobs)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
