"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU tests / benchmark.

This package holds generators and storage-format encoders only - none of the arithmetic of the
operations under test - and imports neither the oracle nor the GPU library.
"""
