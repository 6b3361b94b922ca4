"""MI355X-native packed ViT image encoder: thin Python binding over libvitenc.so.

The binding marshals arguments only; every step of the encoder runs inside the HIP
library.  PyTorch supplies device memory and the stream.
"""
from .binding import (  # noqa: F401
    TokenHandoff,
    VitEncoder,
    VitError,
    lib_path,
    load_library,
    preprocess_tiles,
    vit_encode_packed,
    vit_encode_packed_graph,
    vit_encode_packed_static,
    vit_encoder_create,
    vit_encoder_destroy,
    vit_encoder_query,
    vit_mfma_ceiling,
    vit_preprocess_tiles,
    vit_weight_count,
)
