"""signSGD / Signum with majority vote on one MI355X: thin Python binding over libsignvote.so.

The library (hand-written HIP for gfx950, C ABI in include/signvote.h) does all the work; this
package only marshals torch tensors (device memory + the current stream) into its calls.
There is no CPU fallback: loading fails loudly if the library has not been built
(`python -m paper_1810_05291_amd.build`).
"""
from .binding import (  # noqa: F401
    SSV_F32,
    SSV_BF16,
    SignvoteError,
    library_path,
    load_library,
    words_for,
    sign_pack,
    signum_momentum_pack,
    majority_vote,
    apply_sign_update,
    vote_apply,
    signum_step,
    status_string,
    version,
    bench_copy,
    MultiTensorPlan,
    signum_step_multi,
    multi_workspace,
    SSV_QSGD_L2,
    SSV_QSGD_MAX,
    qsgd_workspace,
    qsgd_norms,
    qsgd_norms_static,
    qsgd_quantize,
    qsgd_aggregate_apply,
)
from .optim import FlatLayout, SignumMajorityVote, SignumMajorityVoteMulti  # noqa: F401,E402
