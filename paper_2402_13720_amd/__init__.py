"""MI355X-native verification step of Ouroboros speculative decoding.

``workloads`` (seeded synthetic inputs) imports without the native library;
``binding`` loads libouro.so and raises if it has not been built.
"""
__all__ = ["workloads", "binding", "build"]
