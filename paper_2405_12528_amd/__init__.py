"""SirLLM memory-retention hot path (token-entropy scoring, decay, sink/top-k/recent selection,
KV compaction) as hand-written HIP kernels for MI355X (gfx950) behind a C ABI.

``paper_2405_12528_amd.binding`` loads the shared library and exposes the entry points of
``include/sirllm.h`` under the same names; it raises at import when the library has not been
built.  ``paper_2405_12528_amd.synth`` holds the seeded synthetic workloads.
"""
__version__ = "0.1.0"
