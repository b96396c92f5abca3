"""MI355X-native SERQ linear layer: HIP kernels behind a C ABI, with a thin ctypes binding.

    from paper_2603_08185_amd import binding as serq
    pk = serq.pack_weights(W, s, r)                 # offline
    Xq, scale = serq.quantize_act(X_hat, pk.s_inv, abits)
    Y = serq.linear(Xq, scale, abits, pk.Wq, pk.wscale, M, N, K, Rp=pk.Rp, r=r)

The shared library is loaded on first use; importing the package never needs a GPU.
"""
from . import binding  # noqa: F401

__all__ = ["binding"]
