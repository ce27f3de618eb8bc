"""Shared helpers of the tests: build one seeded problem for both sides.

The GPU side gets the float32 blob laid out by the table the *library* reports; the oracle gets the
same tensors keyed by the names the *oracle* lists.  Both tables are asserted equal first."""
import numpy as np

from oracle import subnet_eval as E
from workloads import tensors as T


def make_problem(arch, seed, bf16):
    import paper_2306_17266_amd as S
    lib_table = S.sushi_describe_supernet(arch)
    ora_table = E.supernet_tensors(arch)
    assert lib_table == [(n, tuple(s), k) for n, s, k in ora_table]
    tensors = T.make_weights([(s, k) for _, s, k in lib_table], seed, bf16)
    return T.flatten(tensors), E.name_weights(arch, tensors)


def rel_l2(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.linalg.norm(got - want) / np.linalg.norm(want))


def oracle_logits(arch, wts, cfg, x_nhwc):
    return E.forward(arch, wts, cfg, np.ascontiguousarray(x_nhwc.transpose(0, 3, 1, 2)))


def oracle_logits_bf16_stores(arch, wts, cfg, x_nhwc):
    """The oracle's diagnostic variant: every stored feature map rounded to bf16 (nearest even), all
    arithmetic as in the acceptance oracle.  Not the acceptance reference: it shows how much of a
    query's error budget the bf16 activation format alone uses up."""
    return E.forward(arch, wts, cfg, np.ascontiguousarray(x_nhwc.transpose(0, 3, 1, 2)), act_round=T.round_to_bf16)
