"""The whole path under HIP graph capture: every entry point only launches kernels on the
stream it is given, so a step can be captured once and replayed.  Replays are checked bit
for bit against the eager results, several times, with eager work and synchronisations of
the program's own in between and with the outputs cleared before every replay.
"""
import numpy as np
import pytest
import torch

from paper_2311_16883_amd import binding as B
from paper_2311_16883_amd import synth

pytestmark = pytest.mark.gpu


def to_dev(a):
    return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()


class Buffers:
    def __init__(self, spec, seed):
        X, dY = synth.make_pair(spec, seed)
        self.spec = spec
        self.X, self.dY = to_dev(X), to_dev(dY)
        self.n_keep = B.bsr_keep_count(spec.nblocks, spec.keep)
        code = B.dtype_code(self.X.dtype)
        nbytes = max(B.bsr_workspace_bytes(op, spec.M, spec.K, spec.N, spec.br, spec.bc, code)
                     for op in (B.BSR_OP_SCORE_SELECT, B.BSR_OP_COMPRESS, B.BSR_OP_T_DENSE_MATMUL))
        dev = self.X.device
        self.ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
        self.mask = torch.empty(spec.nblocks, dtype=torch.uint8, device=dev)
        self.row_ptr = torch.empty(spec.nbr + 1, dtype=torch.int32, device=dev)
        self.col_idx = torch.empty(self.n_keep, dtype=torch.int32, device=dev)
        self.values = torch.empty((self.n_keep, spec.br, spec.bc), dtype=self.X.dtype, device=dev)
        self.Xhat = torch.empty((spec.M, spec.K), dtype=self.X.dtype, device=dev)
        self.dW = torch.empty((spec.K, spec.N), dtype=torch.float32, device=dev)

    def outputs(self):
        return [self.mask, self.row_ptr, self.col_idx, self.values, self.Xhat, self.dW]

    def clear(self):
        for t in self.outputs():
            t.view(torch.uint8).fill_(0xA5)          # a fill kernel, not a memset node

    def step(self):
        s = self.spec
        B.bsr_score_select(self.X, s.br, s.bc, s.keep, keep_mask=self.mask, ws=self.ws)
        B.bsr_compress(self.X, s.br, s.bc, self.mask, self.n_keep, row_ptr=self.row_ptr,
                       col_idx=self.col_idx, values=self.values, ws=self.ws)
        B.bsr_decompress(self.row_ptr, self.col_idx, self.values, s.M, s.K, s.br, s.bc, out=self.Xhat)
        B.bsr_t_dense_matmul(self.row_ptr, self.col_idx, self.values, s.M, s.K, s.br, s.bc, self.dY,
                             dW=self.dW, ws=self.ws)

    def snapshot(self):
        torch.cuda.synchronize()
        return [t.view(torch.uint8).cpu().numpy().copy() for t in self.outputs()]


@pytest.mark.parametrize("spec", [
    synth.TensorSpec("graph_32", 36864, 384, 512, 32, 32, "bf16", keep=0.5),    # 13824 blocks: grid-wide selection; split-K dW
    synth.TensorSpec("graph_14", 2744, 196, 196, 14, 14, "bf16", keep=0.5),     # zero-filled LDS tiles
], ids=lambda s: s.name)
def test_replays_match_eager(spec):
    a = Buffers(spec, 11)
    other = Buffers(spec, 12)                       # eager work between the replays
    a.clear()
    a.step()
    want = a.snapshot()
    other.step()
    other_want = other.snapshot()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        a.step()
    for rep in range(4):
        a.clear()
        other.clear()
        torch.cuda.synchronize()
        graph.replay()
        other.step()
        got, other_got = a.snapshot(), other.snapshot()
        for w, g in zip(want, got):
            assert w.tobytes() == g.tobytes(), f"replay {rep} differs from the eager result"
        for w, g in zip(other_want, other_got):
            assert w.tobytes() == g.tobytes(), f"eager work after replay {rep} differs"


def test_batched_score_select_replays_match_eager():
    """The several-tensors-per-call entry point under capture: its item array is read on the host
    while the call is recorded, the launches replay with the same arguments."""
    specs = [synth.TensorSpec("g_fc", 36864, 384, 64, 32, 32, "bf16", keep=0.5),       # grid-wide selection
             synth.TensorSpec("g_small", 6272, 384, 64, 32, 32, "bf16", keep=0.25),    # one workgroup
             synth.TensorSpec("g_patch", 2744, 196, 64, 14, 14, "bf16", keep=0.5)]     # LDS-staged scoring
    Xs = [to_dev(synth.make_pair(sp, 21 + i)[0]) for i, sp in enumerate(specs)]
    batch = B.SelectBatch(Xs, [(sp.br, sp.bc) for sp in specs], [sp.keep for sp in specs])
    ws = torch.empty(batch.ws_bytes + 256, dtype=torch.uint8, device="cuda")
    B.bsr_score_select_batched(batch, ws=ws)
    torch.cuda.synchronize()
    want = [m.cpu().numpy().copy() for m in batch.keep_masks]
    for sp, X, w in zip(specs, Xs, want):
        single = B.bsr_score_select(X, sp.br, sp.bc, sp.keep)
        torch.cuda.synchronize()
        assert np.array_equal(single.cpu().numpy(), w)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.bsr_score_select_batched(batch, ws=ws)
    for rep in range(3):
        for m in batch.keep_masks:
            m.fill_(9)
        ws.fill_(0x5A)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for m, w in zip(batch.keep_masks, want):
            assert np.array_equal(m.cpu().numpy(), w), f"replay {rep}"


def test_batched_dw_replays_match_eager():
    specs = [synth.TensorSpec("g_fc1", 6272, 384, 1536, 32, 32, "bf16", keep=0.5),
             synth.TensorSpec("g_fc2", 6272, 1536, 384, 32, 32, "bf16", keep=0.5),
             synth.TensorSpec("g_patch", 5488, 196, 196, 14, 14, "bf16", keep=0.5)]
    problems = []
    for i, sp in enumerate(specs):
        X, dY = synth.make_pair(sp, 31 + i)
        Xd = to_dev(X)
        mask = B.bsr_score_select(Xd, sp.br, sp.bc, sp.keep)
        rp, ci, val = B.bsr_compress(Xd, sp.br, sp.bc, mask, B.bsr_keep_count(sp.nblocks, sp.keep))
        problems.append((rp, ci, val, sp.M, sp.K, sp.br, sp.bc, to_dev(dY)))
    batch = B.MatmulBatch(problems)
    ws = torch.empty(batch.ws_bytes + 256, dtype=torch.uint8, device="cuda")
    B.bsr_t_dense_matmul_batched(batch, ws=ws)
    torch.cuda.synchronize()
    want = [o.cpu().numpy().copy() for o in batch.dWs]
    for pr, w in zip(problems, want):
        single = B.bsr_t_dense_matmul(*pr)
        torch.cuda.synchronize()
        # products that share a launch may split their contraction differently: equal to rounding
        ref = single.cpu().numpy().astype(np.float64)
        assert np.max(np.abs(w - ref)) <= 2e-6 * np.max(np.abs(ref))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.bsr_t_dense_matmul_batched(batch, ws=ws)
    for rep in range(3):
        for o in batch.dWs:
            o.fill_(float("nan"))
        ws.fill_(0x5A)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, w in zip(batch.dWs, want):
            assert o.cpu().numpy().tobytes() == w.tobytes(), f"replay {rep}"


def test_batched_compress_and_decompress_replays_match_eager():
    specs = [synth.TensorSpec("g_fc1", 3136, 384, 1, 32, 32, "bf16", keep=0.5),
             synth.TensorSpec("g_fc2", 3136, 1536, 1, 32, 32, "bf16", keep=0.5),
             synth.TensorSpec("g_patch", 5488, 196, 1, 14, 14, "bf16", keep=0.5)]
    problems = []
    for i, sp in enumerate(specs):
        X, _ = synth.make_pair(sp, 41 + i)
        Xd = to_dev(X)
        mask = B.bsr_score_select(Xd, sp.br, sp.bc, sp.keep)
        problems.append((Xd, sp.br, sp.bc, mask, B.bsr_keep_count(sp.nblocks, sp.keep)))
    cb = B.CompressBatch(problems)
    cws = torch.empty(cb.ws_bytes + 256, dtype=torch.uint8, device="cuda")
    B.bsr_compress_batched(cb, ws=cws)
    db = B.DecompressBatch([(rp, ci, val, sp.M, sp.K, sp.br, sp.bc) for (rp, ci, val), sp in zip(cb.outputs, specs)])
    B.bsr_decompress_batched(db)
    torch.cuda.synchronize()
    want = [[t.view(torch.uint8).cpu().numpy().copy() for t in trio] for trio in cb.outputs]
    want_dense = [o.view(torch.uint8).cpu().numpy().copy() for o in db.outputs]
    for pr, trio, sp, dense in zip(problems, want, specs, want_dense):
        single = B.bsr_compress(*pr)
        back = B.bsr_decompress(*single, sp.M, sp.K, sp.br, sp.bc)
        torch.cuda.synchronize()
        for a, w in zip(single, trio):
            assert a.view(torch.uint8).cpu().numpy().tobytes() == w.tobytes()
        assert back.view(torch.uint8).cpu().numpy().tobytes() == dense.tobytes()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.bsr_compress_batched(cb, ws=cws)
        B.bsr_decompress_batched(db)
    for rep in range(3):
        for trio in cb.outputs:
            for t in trio:
                t.view(torch.uint8).fill_(0x77)
        for o in db.outputs:
            o.view(torch.uint8).fill_(0x77)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for trio, w3 in zip(cb.outputs, want):
            for t, w in zip(trio, w3):
                assert t.view(torch.uint8).cpu().numpy().tobytes() == w.tobytes(), f"replay {rep}"
        for o, w in zip(db.outputs, want_dense):
            assert o.view(torch.uint8).cpu().numpy().tobytes() == w.tobytes(), f"replay {rep}"
