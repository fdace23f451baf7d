"""MI355X-native SubNetAct forward path: Python binding over libsubnetact.so.

Argument marshalling only; every step of the path runs in the HIP kernels behind
the C ABI declared in include/subnetact.h.  Importing this package does not load
the library; the first call does, and fails loudly if it has not been built.
"""
from .binding import (ArchDesc, SubnetCfgC, Supernet, lib, library_path, arch_desc_from_spec,
                      tensor_infos, norm_infos, pack_weights, pack_stats, cfg_to_c,
                      supernet_load, subnet_forward, SnaError)

__all__ = ["ArchDesc", "SubnetCfgC", "Supernet", "lib", "library_path", "arch_desc_from_spec",
           "tensor_infos", "norm_infos", "pack_weights", "pack_stats", "cfg_to_c",
           "supernet_load", "subnet_forward", "SnaError"]
