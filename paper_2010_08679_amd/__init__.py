"""MI355X-native hot path of an incremental, quantized checkpoint encoder for embedding tables
(Check-N-Run, arXiv 2010.08679): touched-row tracking, dirty-row compaction, per-row uniform
quantization with dense packing, and the de-quantize + scatter restore.

``binding`` mirrors the C ABI of ``include/cnr.h`` one to one; ``checkpoint`` owns the device
buffers one table needs and strings the calls together; ``synth`` draws synthetic inputs.
The compute lives in ``csrc/`` (HIP, gfx950) and is reached only through ``libcnr.so``.
"""
from .binding import *  # noqa: F401,F403
from .binding import CnrError, load  # noqa: F401
from .checkpoint import BatchCheckpointer, EncodedRows, HostCheckpointWriter, TableCheckpointer  # noqa: F401
from .autotune import select_greedy_params  # noqa: F401
