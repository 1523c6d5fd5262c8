"""MI355X-native hot path of DCI dual-cache GNN inference (arXiv 2503.01281).

The work is done by ``libdci.so`` (hand-written HIP for gfx950 behind the C boundary declared
in ``include/dci.h``); this package is the thin ctypes binding with the same call names.
PyTorch is used for device / pinned memory and the stream only.
"""
from .binding import (  # noqa: F401
    DCI_MAX_HOPS, KERNEL_CLASSES, STATS_WORDS, STAT, Blocks, Cache, Context, DciError, Graph, blocks_bounds,
    DCI_MODEL_GCN_AVG, DCI_MODEL_SAGE_MEAN, DCI_MODEL_SAGE_SUM, DCI_OPT_LINEAR_KERNEL, DCI_OPT_LINEAR_SPLIT, DCI_OPT_RELABEL_SPIN_LIMIT, DCI_OPT_TEST_RELABEL_FIRST_TICKET, DCI_FILL_ADJ_ELEMENTS, DCI_FILL_STRICT_SPLIT,
    dci_fill_caches, dci_gather_features, dci_gnn_forward, dci_presample_count, dci_sage_forward, dci_sample_khop,
    dci_sample_khop_static, STATIC_SCRATCH_BYTES,
    library_path, load_library, pinned_empty, dci_probe_read, Lane, dci_infer_batches, dci_gather_forward, DCI_OPT_FUSED_INPUT, DCI_OPT_RELABEL_TILE_ITERS, DCI_OPT_INPUT_LAYER,
)
