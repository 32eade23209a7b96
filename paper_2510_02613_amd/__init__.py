"""MI355X-native MoE expert layer of one expert-parallel rank (ElasticMoE hot path).

`binding` mirrors the C ABI of libelasticmoe.so one to one; `layer.MoELayer` is a
small convenience holder of the device buffers (torch is used for memory and
streams only).
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
