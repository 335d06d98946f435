"""GPU test of tfhe_gate_batch_noalloc, the entry point for callers that cannot allocate: its
output ciphertexts must equal, byte for byte, those of tfhe_gate_batch on the same inputs -- on two
calls in a row that share the static scratch array, the second one smaller than the first."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


def test_noalloc_entry_point_equals_gate_batch_on_successive_calls():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    import paper_1806_03461_amd as T
    sk, ck = T.tfhe_keygen(T.default_params(), workloads.KEY_SEED)

    rng = np.random.default_rng(99)
    bits = rng.integers(0, 2, (2, T.NOALLOC_MAX_GATES)).astype(np.uint8)
    a = T.to_device(T.tfhe_encrypt(sk, 71, bits[0]))
    b = T.to_device(T.tfhe_encrypt(sk, 72, bits[1]))

    # before the upload the call refuses (the upload is what allocates and finds the scratch)
    out = torch.zeros_like(a)
    with pytest.raises(T.TfheError) as e:
        T.tfhe_gate_batch_noalloc(ck, "AND", a, b, out, 4)
    assert e.value.code == -2
    T.tfhe_cloud_key_upload(ck)

    # first call: the largest batch the scratch holds; second call: a small, ragged one of another
    # gate kind on other inputs (it finds the first call's samples in the scratch)
    for op, first, count in (("XOR", 0, T.NOALLOC_MAX_GATES), ("NAND", 1000, 37), ("OR", 5, 300)):
        aa, bb = a[first:first + count].contiguous(), b[first:first + count].contiguous()
        want = torch.zeros_like(aa)
        T.tfhe_gate_batch(ck, op, aa, bb, want, count)
        got = torch.zeros_like(aa)
        T.tfhe_gate_batch_noalloc(ck, op, aa, bb, got, count)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (op, count)
        x, y = bits[0][first:first + count], bits[1][first:first + count]
        plain = {"XOR": x ^ y, "NAND": 1 - (x & y), "OR": x | y}[op]
        assert np.array_equal(T.tfhe_decrypt(sk, T.to_host(got)), plain), (op, count)

    # one gate more than the scratch holds: a clear error, nothing enqueued
    big = torch.zeros((T.NOALLOC_MAX_GATES + 1, a.shape[1]), dtype=torch.int32, device="cuda")
    with pytest.raises(T.TfheError) as e:
        T.tfhe_gate_batch_noalloc(ck, "AND", big, big, big, T.NOALLOC_MAX_GATES + 1)
    assert e.value.code == -3 and "at most" in str(e.value)
    T.tfhe_gate_batch_noalloc(ck, "AND", 0, 0, 0, 0)          # count 0: no-op
