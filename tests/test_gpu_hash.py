"""GPU parity for the checkpoint hashes: SHA-256 of FP32 weights in device memory (flat and as a tree
of chunks) and the Merkle root over the leaves, byte for byte against the oracle (hashlib)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import hash_tree as ht

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.fixture(scope="module")
def vt():
    import paper_2403_09603_amd as m
    m.load_library()
    return m


def weights_bytes(nbytes, seed):
    """FP32 weights ~ N(0, 0.02^2) as raw bytes (the tail of an odd length is cut mid-value)."""
    w = si.normal(((nbytes + 3) // 4,), seed, 0.02).astype(np.float32)
    return w.view(np.uint8)[:nbytes].copy()


def gpu_tree(vt, data, chunk):
    d = torch.from_numpy(data).to(DEV) if data.size else torch.empty(0, dtype=torch.uint8, device=DEV)
    out = torch.zeros(32, dtype=torch.uint8, device=DEV)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_SHA256_TREE, 1, data.size, chunk))
    vt.vt_sha256_tree(d, chunk, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy().tobytes()


@pytest.mark.parametrize("nbytes", [0, 1, 3, 55, 56, 63, 64, 65, 119, 120, 128, 1000, 4096, 4097, 65536 + 36, 1 << 20])
def test_flat_sha256(vt, nbytes):
    data = weights_bytes(nbytes, si.seed_for(8, 0) + nbytes)
    assert gpu_tree(vt, data, 0) == ht.sha256(data.tobytes())


@pytest.mark.parametrize("chunk", [64, 128, 1024, 4096])
@pytest.mark.parametrize("nbytes", [0, 1, 64, 65, 100, 4096, 4097, 4096 * 64, 4096 * 64 + 4, 4096 * 65 - 1, (3 << 20) + 52, 64 * 64 * 64 + 32])
def test_tree_sha256(vt, nbytes, chunk):
    data = weights_bytes(nbytes, si.seed_for(8, 1) + nbytes)
    assert gpu_tree(vt, data, chunk) == ht.sha256_tree(data.tobytes(), chunk)


def test_tree_of_a_model_sized_tensor(vt):
    # 25.6 M FP32 weights (ResNet-50's size), chunk 1024: 100 000 chunks, three levels
    data = weights_bytes(25_600_000 * 4, si.seed_for(8, 2))
    got = gpu_tree(vt, data, 1024)
    assert got == ht.sha256_tree(data.tobytes(), 1024)
    # one flipped weight bit changes the digest; the same bytes give the same digest
    data2 = data.copy()
    data2[77_777_777] ^= 1
    assert gpu_tree(vt, data2, 1024) != got
    assert gpu_tree(vt, data, 1024) == got


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 7, 8, 9, 63, 64, 65, 127, 129, 1000, 1001, 4097])
def test_merkle_root(vt, n):
    rng = si.rng(si.seed_for(8, 3) + n)
    leaves = rng.integers(0, 256, (n, 32), dtype=np.uint8)
    d = torch.from_numpy(leaves).to(DEV)
    root = torch.zeros(32, dtype=torch.uint8, device=DEV)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_MERKLE_ROOT, 1, n))
    vt.vt_merkle_root(d, root, ws)
    torch.cuda.synchronize()
    assert root.cpu().numpy().tobytes() == ht.merkle_root([bytes(l) for l in leaves])
    assert np.array_equal(d.cpu().numpy(), leaves)            # the leaves are left as they were


def test_checkpoint_leaves_then_root(vt):
    """Algorithm "train": a leaf per checkpoint from the weights at that step, then the root; a second
    run that differs in one weight at one checkpoint ends with another root, an identical run with the same."""
    n_ckpt, nbytes, chunk = 6, 300_000, 4096
    states = [weights_bytes(nbytes, si.seed_for(8, 4) + c) for c in range(n_ckpt)]

    def run(states):
        leaves = torch.zeros(n_ckpt, 32, dtype=torch.uint8, device=DEV)
        ws = vt.alloc_workspace(max(vt.vt_workspace_bytes(vt.VT_OP_SHA256_TREE, 1, nbytes, chunk),
                                    vt.vt_workspace_bytes(vt.VT_OP_MERKLE_ROOT, 1, n_ckpt)))
        for c, st in enumerate(states):
            vt.vt_sha256_tree(torch.from_numpy(st).to(DEV), chunk, leaves[c], ws)
        root = torch.zeros(32, dtype=torch.uint8, device=DEV)
        vt.vt_merkle_root(leaves, root, ws)
        torch.cuda.synchronize()
        return leaves.cpu().numpy(), root.cpu().numpy().tobytes()

    leaves, root = run(states)
    exp_leaves = [ht.sha256_tree(s.tobytes(), chunk) for s in states]
    assert [bytes(l) for l in leaves] == exp_leaves
    assert root == ht.merkle_root(exp_leaves)
    assert run(states)[1] == root
    tampered = [s.copy() for s in states]
    tampered[3][12345] ^= 0x80
    leaves2, root2 = run(tampered)
    assert root2 != root
    differing = [c for c in range(n_ckpt) if bytes(leaves2[c]) != exp_leaves[c]]
    assert differing == [3]                                   # the leaf the binary search of the game would find
