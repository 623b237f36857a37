"""The two roles of the shared-backbone test, each run as a process of its own (python tests/ipc_roles.py ROLE DIR):

holder -- the "backbone function" of paper section 4.4: puts W0 into a device allocation of its own, exports the
          allocation's IPC handle to DIR/handle.json, waits until every client has reported, checks that W0 is
          bit-for-bit what it wrote, frees it.
client -- a "LoRA function": opens the handle, uses the mapped pointer as W0 of lora_linear with its OWN adapters,
          activations, plan and workspace, compares Y with the oracle, reports to DIR/client_<name>.json.
"""
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

K, N = 1024, 2048  # the backbone weight shared here: 4 MiB of bf16


class _Raw:
    """A device allocation that torch did not make, presented through the CUDA array interface (int16 = bf16 bits)."""

    def __init__(self, ptr, shape):
        self.__cuda_array_interface__ = {"data": (ptr, False), "shape": shape, "typestr": "<i2", "version": 2}


def backbone_workload(seed_x, ids, lens):
    import numpy as np
    from workloads import make_custom
    wl = make_custom(seed=4242, dtype="bf16", K=K, N=N, ranks=(16, 8, 32), scales=(2.0, 1.0, 0.5), req_adapter=ids, req_ntok=lens)
    return wl


def holder(d, n_clients):
    import numpy as np
    import torch
    from paper_2505_14468_amd import binding as B
    wl = backbone_workload(0, [0], [1])
    bits = wl.W0(0)
    ptr = B.lora_backbone_alloc(0, bits.nbytes)
    view = torch.as_tensor(_Raw(ptr, bits.shape), device="cuda")
    view.copy_(torch.from_numpy(bits.view(np.int16)))
    torch.cuda.synchronize()
    handle = B.lora_backbone_export(0, ptr)
    with open(os.path.join(d, "handle.tmp"), "w") as f:
        json.dump({"handle": handle.hex(), "bytes": int(bits.nbytes)}, f)
    os.replace(os.path.join(d, "handle.tmp"), os.path.join(d, "handle.json"))
    print("holder: exported", flush=True)
    t0 = time.time()
    while time.time() - t0 < 150:
        if sum(os.path.exists(os.path.join(d, f"client_{i}.json")) for i in range(n_clients)) == n_clients:
            break
        time.sleep(0.05)
    torch.cuda.synchronize()
    same = bool(torch.equal(view.cpu(), torch.from_numpy(bits.view(np.int16))))
    B.lora_backbone_free(0, ptr)
    with open(os.path.join(d, "holder.json"), "w") as f:
        json.dump({"unchanged": same}, f)
    print("holder: done, W0 unchanged:", same, flush=True)
    return 0 if same else 1


def client(d, name):
    import numpy as np
    import torch
    from paper_2505_14468_amd import binding as B
    from paper_2505_14468_amd import runtime as rt
    from oracle import oracle_workload
    from workloads import to_f64
    t0 = time.time()
    while not os.path.exists(os.path.join(d, "handle.json")):
        if time.time() - t0 > 120:
            return 3
        time.sleep(0.05)
    info = json.load(open(os.path.join(d, "handle.json")))
    ctx = rt.Context(0)
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    t1 = time.perf_counter()
    ptr = B.lora_backbone_open(0, bytes.fromhex(info["handle"]))
    open_ms = (time.perf_counter() - t1) * 1e3
    free1, _ = torch.cuda.mem_get_info()
    W0 = torch.as_tensor(_Raw(ptr, (N, K)), device="cuda").view(torch.bfloat16)  # zero-copy: the holder's memory
    assert W0.data_ptr() == ptr
    rng = np.random.default_rng(int(name) + 1)
    worst = 0.0
    for rep, T_per in enumerate((2, 40)):  # a decode-sized and a prefill-sized batch of this function
        ids = rng.integers(-1, 3, size=6)
        lens = rng.integers(1, T_per + 1, size=6)
        wl = backbone_workload(0, ids, lens)
        wl._cache[("X", 0)] = wl._draw(1, 100 + int(name), rep, (wl.T, K), 1.0)  # this function's own activations
        X, _, table = rt.upload_workload(wl, 0, ctx.device)  # (its own adapters; the uploaded copy of W0 is not used)
        pl = rt.plan(ctx, wl.req_adapter, wl.req_ntok, wl.ranks, wl.r_max)
        Y = rt.linear(ctx, pl, X, W0, table)
        torch.cuda.synchronize()
        assert pl.status(ctx)[0] == 0
        ref = oracle_workload(wl)
        rms = float(np.sqrt((ref ** 2).mean()))
        worst = max(worst, float(np.abs(to_f64(rt.bits_from_tensor(Y)) - ref).max() / rms))
    del W0
    B.lora_backbone_close(0, ptr)
    ctx.close()
    out = {"err_over_rms": worst, "open_ms": open_ms, "device_bytes_taken_by_the_mapping": int(free0 - free1),
           "backbone_bytes": info["bytes"]}
    with open(os.path.join(d, f"client_{name}.json"), "w") as f:
        json.dump(out, f)
    print("client", name, out, flush=True)
    return 0 if worst <= 2e-2 else 2


if __name__ == "__main__":
    role, d = sys.argv[1], sys.argv[2]
    sys.exit(holder(d, int(sys.argv[3])) if role == "holder" else client(d, sys.argv[3]))
