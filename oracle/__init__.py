"""TEST INFRASTRUCTURE -- the CPU oracle (patch-by-patch scanning, fp64).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares no code with the HIP path and imports nothing from it.

  patchscan.c   literal patch-by-patch forward / backward through the original
                strided CNN (paper Sec. 1.1, Fig. 1(a), Sec. 4.3)
  scan.py       ctypes binding + image padding (Sec. 3.3) + high-level helpers
  loss.py       masked softmax cross-entropy and its error map (Sec. 4.3 mask)
  cubescan.c    the same for video: cube-by-cube scanning through the original
                strided 3-D CNN (the extension the paper's closing section proposes)
  cube.py       ctypes binding of cubescan.c + padding of a video
"""
from .scan import (build, pad_image, pack_params, unpack_params, patch_forward,  # noqa: F401
                   STORE_EXACT, STORE_BF16,
                   scan_forward, scan_forward_maps, scan_backward, num_threads, geometry)
from .loss import masked_softmax_xent  # noqa: F401
from .cube import (build3d, pad_video, pack_params3d, unpack_params3d, geometry3d,  # noqa: F401
                   cube_forward_maps, cube_scan_forward, cube_scan_backward)
