"""MI355X-native ShadowKV decode hot path: ctypes binding over the HIP library.

``shadowkv`` (the binding) loads ``libshadowkv.so`` lazily on first use and
raises if it is missing; ``workloads`` draws the synthetic inputs.
"""
__all__ = ["shadowkv"]
