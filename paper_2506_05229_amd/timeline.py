"""Where the time of a grouped-GEMM workgroup goes: a probe, not part of the product path.

    python -m paper_2506_05229_amd.build --timeline            # builds libarmt_hip_timeline.so (-DARMT_GEMM_TIMELINE)
    python -m paper_2506_05229_amd.timeline 1b_32k gate_up     # kinds: qkv, attn_out, gate_up, down, mem_read, ...

The probe library records, for every workgroup of ONE launch of the chosen GEMM kind in the middle of a forward pass
(a step with the full group), the shader clock at its start, after its first k-tile has landed, after its main loop
and after its epilogue, the wall clock at start and end, and the compute unit it ran on.  Printed: cycles per phase,
the gap between consecutive workgroups of a compute unit, and the span of the launch.
"""
import ctypes as C
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))


def main(argv):
    os.environ["ARMT_HIP_LIBRARY"] = os.path.join(HERE, "libarmt_hip_timeline.so")
    sys.path.insert(0, os.path.dirname(HERE))
    import numpy as np
    import torch
    import armt_synth as S
    import paper_2506_05229_amd as P
    name, kind = argv[0], argv[1]
    shape = S.get_shape(name)
    layers, mem_emb = S.make_weights(shape, seed=0)
    model = P.Armt(shape, layers, mem_emb)
    xd = model.embed(S.make_embeddings(shape, seed=0))
    lib = P.load_library()
    lib.armt_timeline_arm.argtypes = [C.c_int32, C.c_int32]
    lib.armt_timeline_read.argtypes = [C.c_void_p, C.c_int64]
    out = model.forward(xd, diagonal=True)
    torch.cuda.synchronize()
    nth = (shape.n_layers + shape.n_segments) // 2            # a launch with the full group
    lib.armt_timeline_arm(P.GEMM_KINDS[kind], nth)
    model.forward(xd, diagonal=True, out=out)
    torch.cuda.synchronize()
    buf = np.zeros(8 * 65536, dtype=np.uint64)
    assert lib.armt_timeline_read(buf.ctypes.data, buf.size) == 0
    r = buf.reshape(-1, 8)
    r = r[r[:, 2] != 0]
    print(f"{name} {kind}: {len(r)} workgroups recorded")
    pro, main_, epi = ((r[:, b] - r[:, a]).astype(np.int64) for a, b in ((2, 3), (3, 4), (4, 5)))
    wall = (r[:, 6] - r[:, 1]).astype(np.int64) * 10          # ns
    q = lambda a: f"mean {a.mean():9.0f}  p10 {np.percentile(a, 10):9.0f}  p50 {np.percentile(a, 50):9.0f}  p90 {np.percentile(a, 90):9.0f}"
    print("  cycles  start -> first k-tile landed:", q(pro))
    print("  cycles  main loop                   :", q(main_))
    print("  cycles  epilogue                    :", q(epi))
    print("  ns      workgroup wall time         :", q(wall), f" (shader clock {(pro + main_ + epi).mean() / wall.mean():.2f} GHz)")
    cu = (r[:, 0] >> np.uint64(32)) * np.uint64(65536) + ((r[:, 0] >> np.uint64(8)) & np.uint64(0xFF))
    gaps, per_cu = [], []
    for c in np.unique(cu):
        m = cu == c
        st, en = np.sort(r[m, 1].astype(np.int64)), np.sort(r[m, 6].astype(np.int64))
        per_cu.append(int(m.sum()))
        gaps += list((st[1:] - en[:-1]) * 10)
    print(f"  {len(per_cu)} compute units, workgroups per unit {min(per_cu)} .. {max(per_cu)}")
    if gaps:
        print("  ns      gap between workgroups of a unit:", q(np.array(gaps)))
    print(f"  launch span {(int(r[:, 6].max()) - int(r[:, 1].min())) * 10 / 1e3:.1f} us")


if __name__ == "__main__":
    main(sys.argv[1:])
