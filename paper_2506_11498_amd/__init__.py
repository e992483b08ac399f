"""MI355X-native hot path of Lag-Relative Sparse Attention: LagKV scoring, per-head top-K
selection and block-sparse causal attention forward/backward, as HIP kernels for gfx950 behind
the C ABI of include/lrsa.h.  This package holds the kernels' sources (csrc/), the build step
and a ctypes binding; `inputs` is the seeded synthetic-input generator."""
from . import inputs  # noqa: F401
from .binding import (IMPL_AUTO, IMPL_COMPACT, IMPL_GENERIC, LrsaError, LrsaParams, lib, lrsa_attn_bwd, lrsa_attn_fwd, lrsa_cache_compress, lrsa_decode_attn, lrsa_decode_attn_static, lrsa_attn_fwd_fill, lrsa_attn_bwd_fill, lrsa_attn_bwd_finish, fill_workspace_bytes,  # noqa: F401
                      lrsa_check_idx, lrsa_score, lrsa_score_select, lrsa_select, make_params, num_scored_chunks, params_for, score_poll_limit, score_route, timing_enable,
                      timing_records, workspace_bytes)
