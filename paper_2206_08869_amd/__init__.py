"""MI355X-native integer-only discrete-flow inference (arXiv 2206.08869).

Python surface = the C ABI of libiodf (include/iodf.h) plus a small convenience
class. Importing the package does not load the library; the first call does, and
raises if it has not been built.
"""
from .binding import (Flow, IodfError, build_library, load_library, iodf_init, iodf_forward, iodf_inverse,
                      iodf_query, iodf_free, iodf_profile_begin, iodf_profile_end, iodf_prior_cf, iodf_encode, iodf_encode_noalloc,
                      iodf_decode, iodf_codec_tables, iodf_tile_patches, iodf_untile_patches, iodf_conv_probe, iodf_conv_probe_timeline, EXPORTS, LIB_PATH,
                      IODF_Q_Z_ELEMS, IODF_Q_CODE_BYTES, IODF_Q_WORKSPACE_BYTES, IODF_Q_MACS_FORWARD,
                      IODF_Q_MACS_INVERSE, IODF_Q_RANGE_ERRORS, IODF_Q_MAX_BATCH, IODF_Q_IMAGE_H, IODF_Q_IMAGE_W,
                      IODF_Q_CONV_LAUNCHES, IODF_Q_WIDE_MACS_FORWARD, IODF_Q_CODEC_HEADER_WORDS, IODF_Q_CODEC_MAX_WORDS,
                      IODF_Q_CODEC_CLAMPED, IODF_Q_CODEC_OVERFLOWS, IODF_Q_CODEC_BROKEN_LANES,
                      IODF_Q_NOALLOC_MAX_BATCH)
