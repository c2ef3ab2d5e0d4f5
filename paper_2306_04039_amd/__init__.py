"""MI355X-native two-stage retrieval (h-indexer + Mixture of Logits): thin binding over libmolret.so."""
from .binding import (  # noqa: F401
    Corpus,
    MolError,
    hindexer_default_lambda,
    hindexer_topk,
    hindexer_workspace_bytes,
    lib_path,
    load_library,
    mol_corpus_pack,
    mol_score,
    mol_topk,
    mol_workspace_bytes,
    profile_enable,
    profile_read,
    quantize_int8,
    HINDEXER_EXACT,
    HINDEXER_PAPER,
)
