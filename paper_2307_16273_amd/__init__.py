"""MI355X tensor-sumcheck prover for zkDL (arXiv 2307.16273): Python binding.

A thin ctypes layer over the C ABI of libzkdl.so (include/zkdl.h), with the same
entry-point names.  It only marshals arguments: every step of a proof runs in
the library's HIP kernels.  PyTorch is used for device memory and the stream.
There is no CPU fallback: if the library is missing, importing the binding's
functions raises.
"""
from .binding import (Context, Transcript, FrTensor, ZkdlError, load_library, library_path,
                      fr_tensor_upload, tensor_wrap_int, mle_partial_eval, sumcheck_product,
                      sumcheck_matmul, sumcheck_matmul_ft, sumcheck_matmul_general, sumcheck_hadamard, reindex_prove,
                      claims_merge_prove, zkrelu_prove, aggregate_prove, update_prove,
                      host_fr_mul, host_scalar_split, selfcheck_constants, EXPORTED_SYMBOLS,
                      CommitKey, hyrax_commit, hyrax_open, hyrax_verify, commit_selfcheck, aggregate_verify)

__all__ = ["Context", "Transcript", "FrTensor", "ZkdlError", "load_library", "library_path",
           "fr_tensor_upload", "tensor_wrap_int", "mle_partial_eval", "sumcheck_product",
           "sumcheck_matmul", "sumcheck_matmul_ft", "sumcheck_matmul_general", "sumcheck_hadamard", "reindex_prove",
           "claims_merge_prove", "zkrelu_prove", "aggregate_prove", "update_prove",
           "host_fr_mul", "host_scalar_split", "selfcheck_constants", "EXPORTED_SYMBOLS",
           "CommitKey", "hyrax_commit", "hyrax_open", "hyrax_verify", "commit_selfcheck", "aggregate_verify"]
