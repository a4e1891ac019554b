"""MI355X-native path signatures in the word basis: thin Python face of libsig_mi355x.so.

Everything is computed by the HIP kernels behind the C ABI in include/sig.h; this package only
marshals arguments.  There is no CPU fallback: without the built library every call raises.
"""
from .binding import (SigError, WindowPlan, WordSet, lib_path, load_library, sig_backward, sig_backward_residual, sig_backward_checkpointed, sig_forward_checkpointed, sig_backward_static, sig_backward_windows, sig_forward,  # noqa: F401
                      sig_forward_windows,
                      sig_probe_fma_tflops, sig_probe_issue_ns, sig_profile_enable, sig_profile_read,
                      sig_leadlag_backward, sig_leadlag_transform, sig_logsig_backward, sig_logsig_forward,
                      sig_wordset_build_logsig, sig_wordset_build, sig_wordset_build_anisotropic,
                      sig_wordset_build_graph, sig_wordset_build_leadlag_sparse, sig_wordset_build_truncated)
