"""MI355X-native hot path of KVShare's Dual-Stage High Deviation (DHD) KV-cache reuse.

The product is ``libkvshare_hip.so`` (hand-written HIP for gfx950 behind the C ABI of
``include/kvs.h``); ``binding`` is its argument-marshalling ctypes wrapper, ``synth`` the
seeded workload generator used by tests and the benchmark, ``build`` the in-tree hipcc build.
Importing the package does not load the library; ``binding.load()`` does.
"""
__all__ = ["binding", "build", "synth"]
