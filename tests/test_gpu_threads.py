"""Several host threads call the library at once, each on its own stream with its own scratch: the
launcher's process-wide state (kernel tables filled on first use, the large-LDS opt-in per kernel, the
scratch registry, the selector's memo) must serve them all, and every result must equal, bit for bit,
what the same call gives alone (results depend on shape and configuration only).  Products are the NT
operation of Eq. 2 and its TNN route (Algorithm 1) checked against the fp64 oracle once."""
import threading

import numpy as np
import pytest

import oracle
from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import inputs as I
from gpu_util import check_gemm

pytestmark = pytest.mark.gpu

SHAPES = [(300, 520, 260), (64, 128, 8192), (1024, 1024, 1024), (130, 70, 2052), (512, 512, 512), (257, 255, 131)]


def _alone(shape, seed):
    import torch
    m, n, k = shape
    A, B = I.nt_operands(m, n, k, seed)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    C_nt = torch.empty((m, n), device="cuda")
    C_tnn = torch.empty((m, n), device="cuda")
    ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
    mt.mtnn_nt(dA, dB, C_nt)
    mt.mtnn_tnn(dA, dB, C_tnn, ws)
    torch.cuda.synchronize()
    return A, B, dA, dB, C_nt.cpu().numpy(), C_tnn.cpu().numpy()


def test_concurrent_host_threads_on_their_own_streams():
    import torch
    base = [_alone(s, 41000 + i) for i, s in enumerate(SHAPES)]
    for (m, n, k), (A, B, _, _, c_nt, c_tnn) in zip(SHAPES, base):
        C, S = oracle.nt_ref(A, B, with_bound=True)
        check_gemm(c_nt, C, S, k, f"alone nt {m}x{n}x{k}")
        check_gemm(c_tnn, C, S, k, f"alone tnn {m}x{n}x{k}")
    nthreads, rounds = 4, 6
    streams = [torch.cuda.Stream() for _ in range(nthreads)]
    for st in streams:
        mt.lend_scratch(st)
    errors = []
    start = threading.Barrier(nthreads)

    def worker(t):
        try:
            torch.cuda.set_device(0)
            st = streams[t]
            outs = []
            start.wait()
            with torch.cuda.stream(st):
                for r in range(rounds):
                    for i, (m, n, k) in enumerate(SHAPES):
                        j = (i + t + r) % len(SHAPES)              # the threads walk the shapes out of step
                        m, n, k = SHAPES[j]
                        _, _, dA, dB, _, _ = base[j]
                        C1 = torch.empty((m, n), device="cuda")
                        C2 = torch.empty((m, n), device="cuda")
                        ws = torch.empty(mt.mtnn_tnn_workspace_bytes(n, k), dtype=torch.uint8, device="cuda")
                        mt.mtnn_nt(dA, dB, C1, stream=st)
                        label = mt.mtnn_auto(dA, dB, C2, ws, stream=st)
                        assert label == mt.mtnn_select(m, n, k)
                        mt.mtnn_tnn(dA, dB, C2, ws, stream=st)
                        outs.append((j, C1, C2, ws))
            st.synchronize()
            for j, C1, C2, _ in outs:
                if C1.cpu().numpy().tobytes() != base[j][4].tobytes():
                    errors.append(f"thread {t}: NT {SHAPES[j]} differs from the call made alone")
                if C2.cpu().numpy().tobytes() != base[j][5].tobytes():
                    errors.append(f"thread {t}: TNN {SHAPES[j]} differs from the call made alone")
        except Exception as e:  # noqa: BLE001  (reported by the main thread)
            errors.append(f"thread {t}: {type(e).__name__}: {e}")

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(nthreads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
    torch.cuda.synchronize()
    for st in streams:
        mt.lend_scratch(st, 0)
    assert not errors, errors[:5]
