"""MI355X-native Sync EASGD hot path (arXiv 1708.02983): Python face of the C-ABI HIP library.

The binding (and with it the shared library) is loaded on first use, so that
``python -m paper_1708_02983_amd.build`` can run before the library exists.
"""
import importlib

_BINDING_NAMES = (
    "EasgdError", "easgd_grad", "easgd_grad_static", "easgd_layer_product", "STATIC_SCRATCH_BYTES", "easgd_mlp_round", "easgd_mlp_round_workspace_bytes", "easgd_grad_workspace_bytes", "easgd_mlp_num_params", "easgd_sync_round",
    "measgd_round", "easgd_sync_round_bf16", "measgd_round_bf16", "measgd_round_bf16v", "sync_sgd_round", "async_easgd_round", "hogwild_easgd_round", "stream_copy", "stream_triad", "stream_mix32", "mfma_probe", "launch_count", "get_option", "set_option", "lib", "version", "LIB_PATH",
    "OPT_UPDATE_BLOCKS_PER_CU", "OPT_UPDATE_NONTEMPORAL", "OPT_UPDATE_GROUPS", "OPT_GEMM_TILE", "OPT_ROUND_OVERLAP", "OPT_GEMM_XCD", "OPT_GEMM_PAIR", "OPT_MLP_HEAD", "OPT_UPDATE_LAYOUT", "OPT_ROUND_SINGLE_LAUNCH", "OPT_ROUND_SPIN_LIMIT", "round_barrier_timeouts",
)
__all__ = list(_BINDING_NAMES) + ["BatchFeeder"]


def __getattr__(name):
    # the first use of a name imports its module and keeps the object in this module's namespace, so that later
    # uses are plain attribute look-ups (a look-up through the import machinery costs several microseconds, which
    # is a third of a small round's time on the device)
    if name == "BatchFeeder":
        value = importlib.import_module(".feeder", __name__).BatchFeeder
    elif name in _BINDING_NAMES or name == "binding":
        mod = importlib.import_module(".binding", __name__)
        value = mod if name == "binding" else getattr(mod, name)
    else:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
    globals()[name] = value
    return value
