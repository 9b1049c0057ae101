"""Host-side behaviour that needs no GPU: the benchmark's argument handling and the shape of the workload specs."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_refuses_a_multi_rank_launch():
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, env=env,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_workload_specs_match_the_benchmark_definition():
    import json
    from paper_2603_25463_amd import workloads as wl
    cfgs = json.load(open(os.path.join(ROOT, "BASELINE.json")))["configs"]
    assert len(cfgs) == 5 and sorted(wl.SPECS) == [1, 2, 3, 4, 5]
    shapes = {1: (256, 16384, 4), 2: (2048, 16384, 8), 3: (16384, 16384, 8), 4: (32768, 8192, 16), 5: (32768, 65536, 8)}
    for k, (rows, vocab, window) in shapes.items():
        s = wl.SPECS[k]
        assert (s.rows, s.vocab, s.window) == (rows, vocab, window)


def test_small_workload_and_radius_are_seeded_and_well_formed():
    import torch
    from paper_2603_25463_amd import workloads as wl
    a = wl.make(1, device="cpu", rows=64)
    b = wl.make(1, device="cpu", rows=64)
    assert torch.equal(a.draft, b.draft) and torch.equal(a.target, b.target) and torch.equal(a.ids, b.ids)
    assert a.draft.shape == (64, 16384) and a.draft.dtype == torch.float32
    assert int(a.ids.min()) >= 0 and int(a.ids.max()) < 16384
    assert float(a.u_accept.min()) >= 0.0 and float(a.u_accept.max()) < 1.0
    r1, r2 = wl.make_radius(a), wl.make_radius(b)
    assert torch.equal(r1, r2) and r1.shape == a.draft.shape and r1.dtype == a.draft.dtype
    assert torch.isfinite(r1).all() and abs(float(r1.mean())) < 1.5


def test_workload_with_another_number_of_images():
    """`images` changes the batch size of a recipe and nothing else (bench.py's `sustained` entry and --images)."""
    import torch
    from paper_2603_25463_amd import workloads as wl
    a = wl.make(2, device="cpu", rows=512, images=2)
    b = wl.make(2, device="cpu", rows=512, images=2)
    assert a.spec.images == 2 and a.spec.rows == 512 and a.spec.vocab == 16384 and a.spec.window == 8
    assert a.draft.shape == (512, 16384) and a.draft.dtype == torch.float32
    assert torch.equal(a.draft, b.draft) and torch.equal(a.ids, b.ids)
    # the recipe's structure: peaked rows come in aligned 4 x 4 blocks of the 16 x 16 grid
    pk = torch.from_numpy(a.peaked).reshape(2, 4, 4, 4, 4)        # image, block row, row in block, block col, col in block
    assert (pk == pk[:, :, :1, :, :1]).all()
    assert wl.make(2, device="cpu", rows=8, images=8).spec is wl.SPECS[2]
