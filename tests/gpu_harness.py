"""Helpers for the GPU parity tests (the package's own device-side harness)."""
from paper_2604_23108_amd.device_layer import DeviceLayer, from_dev, to_dev  # noqa: F401
