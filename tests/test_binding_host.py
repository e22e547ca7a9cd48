"""The Python binding refuses, on the host and before the library is called, every tensor that would turn
into an out-of-bounds or misinterpreted device access: wrong element count, dtype, stride or device.  No GPU
is needed: the refusals come before any pointer is taken."""
import pytest
import torch

from paper_2601_02360_amd import binding as B


class FakePlan:
    """What Tensors / Messages read from a plan before they call the library."""
    numels = [4096, 10, 0]
    kappa = 32
    quant = True
    num_chunks = 2
    handle = None


def good(n, dtype=torch.float32):
    return torch.zeros(n, dtype=dtype)


def test_tensor_lists_are_checked_against_the_plan():
    plan = FakePlan()
    with pytest.raises(ValueError, match="2 tensors"):
        B.Tensors(plan, [good(4096), good(10)])
    with pytest.raises(ValueError, match="4095 elements"):
        B.Tensors(plan, [good(4095), good(10), None])
    with pytest.raises(ValueError, match="dtype"):
        B.Tensors(plan, [good(4096, torch.float64), good(10), None])
    with pytest.raises(ValueError, match="dtype"):
        B.Tensors(plan, [good(4096), good(10), None], dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="not contiguous"):
        B.Tensors(plan, [torch.zeros(8192)[::2], good(10), None])
    with pytest.raises(ValueError, match="missing"):
        B.Tensors(plan, [good(4096), None, None])
    with pytest.raises(ValueError, match="set 1"):
        B.Tensors(plan, [[good(4096), good(10), None], [good(4096), good(11), None]])
    with pytest.raises(ValueError, match="not on a GPU"):          # everything else is right: the device is not
        B.Tensors(plan, [good(4096), good(10), good(0)])


def test_message_buffers_are_checked_against_the_plan():
    plan = FakePlan()
    with pytest.raises(ValueError, match="pair buffers"):
        B.Messages(plan, [good(64, torch.int16)], [])
    with pytest.raises(ValueError, match="pairs of replica 0"):
        B.Messages(plan, [good(63, torch.int16)], [good(4)])
    with pytest.raises(ValueError, match="levels/values of replica 1"):
        B.Messages(plan, [good(64, torch.int16)] * 2, [good(4), good(64)])
    with pytest.raises(ValueError, match="dtype"):
        B.Messages(plan, [good(64, torch.int32)], [good(4)])


def test_matrix_wrappers_check_shapes_before_the_call():
    x, u, out = torch.zeros(8, 16), torch.zeros(16, 4), torch.zeros(8, 4)
    with pytest.raises(ValueError, match="u"):
        B.sparseloco_subspace_project(x, torch.zeros(15, 4), out)
    with pytest.raises(ValueError, match="projected"):
        B.sparseloco_subspace_project(x, u, torch.zeros(8, 5))
    with pytest.raises(ValueError, match="token_ids"):
        B.sparseloco_subspace_project(x, u, out, t_perp=torch.zeros(5, 16))
    with pytest.raises(ValueError, match="token_ids"):
        B.sparseloco_subspace_project(x, u, out, t_perp=torch.zeros(5, 16), token_ids=torch.zeros(7, dtype=torch.int32))
    with pytest.raises(ValueError, match="token_ids"):
        B.sparseloco_subspace_project(x, u, out, t_perp=torch.zeros(5, 16), token_ids=torch.zeros(8, dtype=torch.int64))
    with pytest.raises(ValueError, match="t_perp"):
        B.sparseloco_subspace_project(x, u, out, t_perp=torch.zeros(5, 15), token_ids=torch.zeros(8, dtype=torch.int32))
    with pytest.raises(ValueError, match="pos_embed"):
        B.sparseloco_subspace_reconstruct(out, u, x, pos_embed=torch.zeros(3, 17))
    with pytest.raises(ValueError, match="activations"):
        B.sparseloco_subspace_reconstruct(out, u, torch.zeros(8, 16, dtype=torch.float64))
    with pytest.raises(ValueError, match="t_perp"):
        B.sparseloco_reproject_embedding(x, torch.zeros(8, 15), torch.zeros(16, 4), torch.zeros(32))
    with pytest.raises(ValueError, match="GPU"):                    # all shapes right, tensors on the host
        B.sparseloco_reproject_embedding(x, x.clone(), torch.zeros(16, 4), torch.zeros(32))


def test_stream_probe_arguments():
    L = B.lib()
    assert L.sparseloco_stream_probe(9, None, None, None, None, 4096, None) == B.SPLC_EINVAL
    assert L.sparseloco_stream_probe(B.SPLC_STREAM_COPY, None, None, None, None, 4096, None) == B.SPLC_EINVAL
    assert L.sparseloco_stream_probe(B.SPLC_STREAM_WRITE, None, None, 4096, None, 100, None) == B.SPLC_EINVAL   # n % 4096
    assert L.sparseloco_stream_probe(B.SPLC_STREAM_WRITE, None, None, 4100, None, 4096, None) == B.SPLC_EALIGN
    assert L.sparseloco_stream_probe(B.SPLC_STREAM_WRITE, None, None, 4096, None, 0, None) == B.SPLC_OK
    shaped = L.sparseloco_stream_probe_shaped
    assert shaped(B.SPLC_STREAM_WRITE, None, None, 4096, None, 4096 * 8, 2, 0, 0, None) == B.SPLC_EINVAL     # slots: 1 or 4
    assert shaped(B.SPLC_STREAM_WRITE, None, None, 4096, None, 4096 * 8, 4, 0, 9, None) == B.SPLC_EINVAL     # groups per unit
    assert shaped(B.SPLC_STREAM_WRITE, None, None, 4096, None, 4096 * 8, 4, -1, 0, None) == B.SPLC_EINVAL
    assert shaped(B.SPLC_STREAM_WRITE, None, None, 4096, None, 4096 * 12, 4, 1, 0, None) == B.SPLC_EINVAL    # 12 groups: no whole runs
    assert shaped(B.SPLC_STREAM_WRITE, None, None, 4096, None, 4096 * 16, 1, 16, 0, None) == B.SPLC_EINVAL   # 64 groups < 8 * 16
    assert shaped(B.SPLC_STREAM_WRITE, None, None, 4096, None, 0, 1, 16, 1, None) == B.SPLC_OK
