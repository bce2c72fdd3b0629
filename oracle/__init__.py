"""CPU oracle for direct sparse convolution (test infrastructure; never on the product path)."""
from .oracle import (build, epilogue, dense_conv, dense_from_csr, sparse_conv, sparse_conv_steps,
                     num_threads, out_shape, quantise_pow2)

__all__ = ["build", "epilogue", "dense_conv", "dense_from_csr", "sparse_conv", "sparse_conv_steps",
           "num_threads", "out_shape", "quantise_pow2"]
