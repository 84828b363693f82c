"""Helpers for the GPU parity tests: the package's device-side harness with out-of-bounds canaries
(guard bands around every output tensor) switched on."""
from paper_2604_23108_amd.device_layer import DeviceLayer as _DeviceLayer, GuardBands, from_dev, to_dev  # noqa: F401


class DeviceLayer(_DeviceLayer):
    def __init__(self, w, inp, training=None, backward=False, guard=True, **cfg_kw):
        super().__init__(w, inp, training=training, backward=backward, guard=guard, **cfg_kw)
