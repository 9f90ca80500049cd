"""MI355X-native Spark-FFN sparse decode path (Spark Transformer, arXiv 2506.06644).

``paper_2506_06644_amd.binding`` exposes the C ABI of ``include/spark.h`` with the same
names; every step of the path runs in the hand-written HIP kernels of ``csrc/``.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    SparkError,
    ffn_workspace_bytes,
    load_library,
    normal_quantile,
    spark_ffn_decode,
    spark_ffn_decode_layers,
    spark_ffn_dense_decode,
    spark_stat_topk,
)
