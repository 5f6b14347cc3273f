"""Pins of the layout oracle: explicit index loops, torch's channels-last storage, and the statistic's independence of storage."""
import numpy as np
import torch

import oracle
from oracle import layout
from paper_2002_06015_amd import workloads as wl


def test_every_element_lands_where_the_definition_says():
    x = np.arange(2 * 3 * 4 * 5, dtype=np.float32).reshape(2, 3, 4, 5)        # [N, H, W, C]
    y = layout.nhwc_to_nchw(x)
    assert y.shape == (2, 5, 3, 4)
    for n in range(2):
        for h in range(3):
            for w in range(4):
                for c in range(5):
                    assert y[n, c, h, w] == x[n, h, w, c]


def test_torch_channels_last_storage_is_the_nhwc_tensor():
    """A torch tensor in channels_last memory format stores [N, H, W, C]; read back through its NCHW view."""
    t = torch.randn(3, 6, 5, 7)                                               # logical NCHW
    cl = t.contiguous(memory_format=torch.channels_last)
    stored = cl.permute(0, 2, 3, 1)                                            # a view of the storage order
    assert stored.is_contiguous()
    assert np.array_equal(layout.nhwc_to_nchw(stored.numpy()), t.numpy())


def test_bits_are_preserved_for_two_byte_elements():
    x = np.random.default_rng(0).integers(0, 65536, size=(2, 3, 3, 4)).astype(np.uint16)
    y = layout.nhwc_to_nchw(x)
    assert y.dtype == np.uint16 and sorted(y.ravel().tolist()) == sorted(x.ravel().tolist())


def test_factor_of_a_conv_layer_does_not_depend_on_the_storage_order():
    """A from the NHWC-stored activations, converted, equals A from the NCHW tensor the generator makes."""
    L = wl.conv_layer(3, 5, 4, 3, 1, 1, 6)
    act = wl.make_act(L, 77)                                                   # [N, C, H, W]
    nhwc = np.ascontiguousarray(act.transpose(0, 2, 3, 1))
    assert np.array_equal(oracle.factor_A(tuple(L), layout.nhwc_to_nchw(nhwc)), oracle.factor_A(tuple(L), act))
