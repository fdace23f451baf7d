"""CPU oracle of the SubNetAct forward path -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It is independent of the HIP library: no shared kernels,
headers, helpers or tables, and neither imports the other.

  inplace.forward             subnet served in place on the max-size tensors
                              (LayerSelect / WeightSlice / SubnetNorm as stated)
  inplace.calibrate           the same forward filling the subnet's SubnetNorm
                              mean / variance rows from the batch it sees
  standalone.extract_subnet,
  standalone.standalone_forward   the definition: copy the slices out, run the
                              resulting ordinary network with library ops
  brute                       definitional nested loops for tiny inputs

Pins (tests marked "not gpu"): brute force vs the C sums, PyTorch CPU library
ops vs the C sums, in place == extracted (every family), max cfg == full
SuperNet, skipped block == identity, SubnetNorm closed forms, activation and
rounding closed forms.  Whole-network logits have no published values to pin
against: the paper prints none.
"""
from . import primitives, inplace, standalone, brute
from .inplace import forward, calibrate
from .standalone import extract_subnet, standalone_forward

__all__ = ["primitives", "inplace", "standalone", "brute", "forward", "calibrate",
           "extract_subnet", "standalone_forward"]
